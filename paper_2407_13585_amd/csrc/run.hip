// Runner: maps every cluster of a clustering onto a kernel instance and
// launches it.  One instance per cluster (an instance is one kernel, in one case two
// kernels in a row); no host synchronisation.
#include "run.hpp"

#include <algorithm>
#include <cstring>
#include <map>
#include <set>

#include "registry.hpp"

namespace fc {

namespace {

struct Builder {
  const Model &m;
  const Clustering &c;
  const std::vector<int> &members;   // nodes of the cluster
  std::set<int> in_cluster;
  std::vector<int> externals;        // node ids, in order of first appearance
  KArgs args;
  int slots = 0;
  std::string err;
  // the same element programs as code for the interpreting kernel (see expr.hpp, Code)
  int n_code = 0, on_stack = 0, gathers = 0;
  bool code_ok = true;               // fits kMaxCode, the value stack and the nesting of gathers

  void emit(unsigned char op, int a = 0, int b = 0, int c = 0) {
    if (n_code >= kMaxCode - 1) { code_ok = false; return; }   // the last entry stays kCodeEnd
    args.code[n_code++] = Code{op, (unsigned char)a, (unsigned char)b, (unsigned char)c};
    switch (op) {
      case kCodeIn: case kCodeGen: ++on_stack; break;
      case kCodeMap: on_stack -= c - 1; break;
      case kCodeEnter: --on_stack; if (++gathers > kInterpGathers) code_ok = false; break;
      case kCodeLeave: --gathers; break;
      case kCodeDup: ++on_stack; break;
      default: --on_stack; break;                              // store, fold, yield
    }
    if (on_stack > kInterpDepth + 1 || on_stack < 0) code_ok = false;
  }

  Builder(const Model &m_, const Clustering &c_, const std::vector<int> &mem)
      : m(m_), c(c_), members(mem), in_cluster(mem.begin(), mem.end()) {
    std::memset(&args, 0, sizeof(args));
  }

  bool fail(const std::string &s) { if (err.empty()) err = s; return false; }

  int external(int a) {
    for (size_t k = 0; k < externals.size(); ++k) if (externals[k] == a) return (int)k;
    externals.push_back(a);
    return (int)externals.size() - 1;
  }

  bool slot_for(int a) {
    if (slots >= kMaxSlots) return fail("element program too large");
    Slot &s = args.p[slots++];
    const fc_node &nd = m.nodes[a];
    s.f[0] = nd.fparam[0]; s.f[1] = nd.fparam[1];
    s.i[0] = nd.iparam[0]; s.i[1] = nd.iparam[1];
    s.ext[0] = (int)nd.shape[0]; s.ext[1] = (int)nd.shape[1];
    if (nd.kind == FC_MAP && nd.fn == FC_FN_MOD_EQ) mod_eq_constants(s);
    if (nd.kind == FC_GENERATE && (nd.fn == FC_FN_CLAMP_SHIFT_2D || nd.fn == FC_FN_ROW_OF_2D)) div_constants(s, s.ext[1]);
    return true;
  }

  // Element program number n_roots of a cluster whose consumer is not elementwise: its
  // signature goes to `sig` as always; `any` receives the signature of the instance that
  // takes any element program of this type (it runs the code between root[k] and the yield).
  int n_roots = 0;
  bool root(int a, std::string &sig, std::string &any) {
    if (n_roots >= kMaxRoots || n_code > 255) code_ok = false; else args.root[n_roots] = (unsigned char)n_code;
    ++n_roots;
    if (!expr(a, sig)) return false;
    emit(kCodeYield);
    any += m.nodes[a].dtype == FC_F32 ? "*f32" : "*i32";
    return true;
  }

  // element program that yields array `a` at the current iteration index
  bool expr(int a, std::string &sig) {
    const fc_node &nd = m.nodes[a];
    const int slot = slots;
    if (!slot_for(a)) return false;
    if (!in_cluster.count(a)) {
      int k = external(a);
      if (k >= kMaxIn - 1) return fail("too many external arrays");
      sig += "in" + std::to_string(k) + (nd.dtype == FC_F32 ? ":f32" : ":i32");
      emit(kCodeIn, k);
      return true;
    }
    switch (nd.kind) {
      case FC_MAP:
        sig += "map" + std::to_string(nd.fn) + "(";
        for (int k = 0; k < nd.nargs; ++k) {
          if (k) sig += ",";
          if (!expr(nd.arg[k], sig)) return false;
        }
        sig += ")";
        emit(kCodeMap, nd.fn, slot, nd.nargs);
        return true;
      case FC_GENERATE:
        sig += "gen" + std::to_string(nd.fn);
        emit(kCodeGen, nd.fn, slot);
        return true;
      case FC_GATHER:
        sig += "gather(";
        if (!expr(nd.arg[0], sig)) return false;
        sig += ",";
        emit(kCodeEnter);
        if (!expr(nd.arg[1], sig)) return false;
        emit(kCodeLeave);
        sig += ")";
        return true;
      default:
        return fail("node " + std::to_string(a) + " cannot be evaluated inside an element program");
    }
  }
};

const char *op_name(int fn, int dtype) {
  if (dtype == FC_F32) return fn == FC_OP_ADD ? "add.f32" : fn == FC_OP_MAX ? "max.f32" : "mul.f32";
  return fn == FC_OP_ADD ? "add.i32" : fn == FC_OP_MAX ? "max.i32" : "mul.i32";
}

}  // namespace

int plan_cluster(const Model &m, const Clustering &c, const std::vector<int> &members, ClusterLaunch &out,
                 std::string &err) {
  Builder b(m, c, members);
  out = ClusterLaunch();
  auto unsupported = [&](const std::string &s) { err = s + (b.err.empty() ? "" : ": " + b.err); return FC_E_UNSUPPORTED; };

  std::vector<int> scans, scatters, folds, foldsegs, stores, forces;
  for (int a : members) {
    const fc_node &nd = m.nodes[a];
    switch (nd.kind) {
      case FC_SCANL: case FC_SCANR: scans.push_back(a); break;
      case FC_SCATTER: scatters.push_back(a); break;
      case FC_FOLD: folds.push_back(a); break;
      case FC_FOLDSEG: foldsegs.push_back(a); break;
      case FC_FORCE: forces.push_back(a); break;
      default:
        if (!c.fused_away[a]) stores.push_back(a);
    }
  }
  std::string sig;
  int n = -1;
  std::string any;                    // signature of the instance that takes any element program, if the shape has one
  bool interpretable = false, reducer_ok = true;
  auto reducer_code = [&](int fn, int dtype) {
    if (dtype == FC_F32) return fn == FC_OP_ADD ? (int)kFoldAddF32 : fn == FC_OP_MAX ? (int)kFoldMaxF32 : (int)kFoldMulF32;
    if (fn == FC_OP_MUL) reducer_ok = false;             // no compiled reducer either
    return fn == FC_OP_ADD ? (int)kFoldAddI32 : (int)kFoldMaxI32;
  };
  auto set_n = [&](int64_t v) { if (n >= 0 && n != (int)v) return false; n = (int)v; return true; };
  auto shape_from = [&](int a) { out.h = (int)m.nodes[a].shape[0]; out.w = (int)m.nodes[a].shape[1]; };

  if (!forces.empty()) {
    if (members.size() != 1) return unsupported("force shares a cluster");
    out.kind = ClusterLaunch::Alias;
    out.alias_of = m.nodes[forces[0]].arg[0];
    out.alias_node = forces[0];
    out.sig = "alias";
    return FC_OK;
  }
  if (!scans.empty()) {
    const int sc = scans[0];
    const int x = m.nodes[sc].arg[0];
    // the scanned array may be a result as well (it is then stored by the same kernel); nothing else is stored
    const bool stores_input = stores.size() == 1 && stores[0] == x;
    if (scans.size() != 1 || scatters.size() > 1 || folds.size() > 1 || !foldsegs.empty() || (!stores.empty() && !stores_input))
      return unsupported("scan cluster shape");
    if (m.nodes[sc].dtype != FC_I32 && (!scatters.empty() || !folds.empty() || c.fused_away[sc]))
      return unsupported("a scan of f32 can be stored, with or without the array it scans, and nothing more");
    // a two-dimensional array is scanned row by row (one row: the same as one dimension)
    const bool by_rows = m.nodes[sc].rank == 2 && m.nodes[sc].shape[0] != 1;
    if (by_rows && (!scatters.empty() || !folds.empty() || c.fused_away[sc]))
      return unsupported("a row scan can be stored, with or without the array it scans, and nothing more");
    sig = by_rows ? (m.nodes[sc].kind == FC_SCANR ? "rowscanr[" : "rowscan[")
                  : (m.nodes[sc].kind == FC_SCANR ? "scanr[" : "scan[");
    any = sig;
    if (by_rows) out.aux = (int)m.nodes[sc].shape[0];
    if (!b.root(x, sig, any)) return unsupported("scan input");
    sig += "]";
    any += "]";
    set_n(m.size(sc));
    shape_from(sc);
    if (!c.fused_away[sc]) { sig += "+offs"; any += "+offs"; out.out_nodes[1] = sc; }
    if (!scatters.empty()) {
      const fc_node &st = m.nodes[scatters[0]];
      if (st.fn != FC_OP_OVERWRITE || st.arg[1] != sc || st.nargs != 4 || st.arg[3] != x)
        return unsupported("scatter fused with a scan must take the scan as index and the scanned flags as flag");
      sig += "+scatter[";
      any += "+scatter[";
      if (!b.root(st.arg[2], sig, any)) return unsupported("scatter value");
      sig += "]";
      any += "]";
      out.out_nodes[0] = scatters[0];
    }
    if (!folds.empty()) {
      const fc_node &f = m.nodes[folds[0]];
      if (f.fn != FC_OP_ADD || f.arg[0] != x || f.shape[0] != 1) return unsupported("fold beside a scan must be (+) over the scanned array");
      sig += "+count";
      any += "+count";
      out.out_nodes[2] = folds[0];
    }
    if (stores_input) {
      sig += "+input";
      any += "+input";
      out.out_nodes[3] = x;
    }
  } else if (!scatters.empty()) {
    if (scatters.size() != 1 || !folds.empty() || !foldsegs.empty() || !stores.empty())
      return unsupported("scatter cluster shape");
    const fc_node &st = m.nodes[scatters[0]];
    sig = st.fn == FC_OP_ADD ? "scatter.add[" : "scatter[";
    any = sig;
    if (!b.root(st.arg[1], sig, any)) return unsupported("scatter index");
    sig += ",";
    any += ",";
    if (!b.root(st.arg[2], sig, any)) return unsupported("scatter value");
    sig += ",";
    any += ",";
    if (st.nargs == 4) {
      if (!b.root(st.arg[3], sig, any)) return unsupported("scatter flag");
    } else {
      sig += "1";
      any += "1";
    }
    sig += "]";
    any += "]";
    set_n(m.size(st.arg[1]));
    shape_from(st.arg[1]);
    out.out_nodes[0] = scatters[0];
  } else if (!foldsegs.empty()) {
    if (foldsegs.size() != 1 || !folds.empty() || !stores.empty()) return unsupported("foldSeg cluster shape");
    const fc_node &f = m.nodes[foldsegs[0]];
    sig = std::string("foldseg.") + op_name(f.fn, f.dtype) + "[";
    any = sig;
    if (!b.root(f.arg[0], sig, any)) return unsupported("foldSeg values");
    sig += "]";
    any += "]";
    set_n(m.size(f.arg[0]));
    shape_from(f.arg[0]);
    out.aux = (int)f.shape[0];
    out.offsets_node = f.arg[1];
    out.out_nodes[0] = foldsegs[0];
  } else if (!folds.empty() && m.nodes[m.nodes[folds[0]].arg[0]].rank == 2 &&
             m.nodes[m.nodes[folds[0]].arg[0]].shape[0] > 1 &&
             m.nodes[folds[0]].shape[0] == m.nodes[m.nodes[folds[0]].arg[0]].shape[0]) {
    // folds over the innermost dimension: one or two reducers over the same argument,
    // optionally consumed by a gather that picks the row
    if (folds.size() > 2 || stores.size() > 1) return unsupported("row-fold cluster shape");
    const fc_node &f0 = m.nodes[folds[0]];
    const int arg = f0.arg[0];
    if (folds.size() == 2 && (m.nodes[folds[1]].arg[0] != arg || m.nodes[folds[1]].dtype != f0.dtype))
      return unsupported("two row folds must reduce the same array");
    sig = std::string("rowfold.") + op_name(f0.fn, f0.dtype);
    if (folds.size() == 2) sig += std::string("+") + op_name(m.nodes[folds[1]].fn, m.nodes[folds[1]].dtype);
    sig += "[";
    any = sig;
    if (!b.root(arg, sig, any)) return unsupported("row-fold argument");
    sig += "]";
    any += "]";
    out.w = (int)m.nodes[arg].shape[1];
    out.h = (int)m.nodes[arg].shape[0];
    if (!stores.empty()) {
      const fc_node &g = m.nodes[stores[0]];
      if (g.kind != FC_GATHER || folds.size() != 1 || g.arg[1] != folds[0] || !c.fused_away[folds[0]])
        return unsupported("a row fold can only be consumed by a gather inside its cluster");
      sig += "@gather(";
      any += "@gather(";
      if (!b.root(g.arg[0], sig, any)) return unsupported("row index");
      sig += ")";
      any += ")";
      n = (int)m.size(stores[0]);
      out.out_nodes[0] = stores[0];
    } else {
      for (int f : folds) if (c.fused_away[f]) return unsupported("row fold consumed inside its cluster");
      n = (int)f0.shape[0];
      out.out_nodes[0] = folds[0];
      if (folds.size() == 2) out.out_nodes[1] = folds[1];
    }
    out.aux = n;
  } else {
    // stored arrays and folds of the flattened argument; compiled instances exist for some of these
    // shapes (at most one fold), the interpreting kernel takes the others (at most kInterpFolds folds)
    if (folds.size() > (size_t)kInterpFolds || (stores.empty() && folds.empty()) || stores.size() + folds.size() > (size_t)kMaxOut)
      return unsupported("cluster with " + std::to_string(stores.size()) + " stored arrays and " + std::to_string(folds.size()) + " folds");
    // the code computes an array once, however many of the cluster's stores and folds take it:
    // after its element program come its consumers, a copy of the value for all but the last
    auto emit_consumers = [&](int array) {
      std::vector<Code> ops;
      for (size_t k = 0; k < stores.size(); ++k)
        if (stores[k] == array) ops.push_back(Code{kCodeStore, (unsigned char)k, 0, 0});
      for (size_t f = 0; f < folds.size(); ++f)
        if (m.nodes[folds[f]].arg[0] == array)
          ops.push_back(Code{kCodeFold, (unsigned char)(stores.size() + f),
                             (unsigned char)reducer_code(m.nodes[folds[f]].fn, m.nodes[folds[f]].dtype), (unsigned char)f});
      for (size_t k = 0; k < ops.size(); ++k) {
        if (k + 1 < ops.size()) b.emit(kCodeDup);
        b.emit(ops[k].op, ops[k].a, ops[k].b, ops[k].c);
      }
    };
    std::set<int> computed;
    for (size_t k = 0; k < stores.size(); ++k) {
      if (k) sig += "+";
      sig += "store[";
      if (!b.expr(stores[k], sig)) return unsupported("stored array");
      sig += "]";
      emit_consumers(stores[k]);
      computed.insert(stores[k]);
      if (!set_n(m.size(stores[k]))) return unsupported("iteration sizes differ inside a cluster");
      if (k == 0) shape_from(stores[0]);
      out.out_nodes[k] = stores[k];
    }
    for (size_t f = 0; f < folds.size(); ++f) {
      const fc_node &fd = m.nodes[folds[f]];
      if (!stores.empty() || f) sig += "+";
      sig += std::string("fold.") + op_name(fd.fn, fd.dtype) + "[";
      const int code_before = b.n_code, stack_before = b.on_stack;
      if (!b.expr(fd.arg[0], sig)) return unsupported("fold argument");
      sig += "]";
      if (computed.count(fd.arg[0])) {   // its code stands where the array was first computed (signature and slots keep both)
        for (int k = code_before; k < b.n_code; ++k) b.args.code[k] = Code{kCodeEnd, 0, 0, 0};
        b.n_code = code_before;
        b.on_stack = stack_before;
      } else {
        emit_consumers(fd.arg[0]);
        computed.insert(fd.arg[0]);
      }
      if (!set_n(m.size(fd.arg[0]))) return unsupported("iteration sizes differ inside a cluster");
      if (stores.empty() && f == 0) shape_from(fd.arg[0]);
      out.out_nodes[stores.size() + f] = folds[f];
    }
    interpretable = b.code_ok && b.on_stack == 0 && reducer_ok;
  }
  // every member must have been reached by an element program or be a root
  out.kind = ClusterLaunch::Kernel;
  out.sig = sig;
  out.args = b.args;
  out.args.n = n;
  out.args.h = out.h;
  out.args.w = out.w;
  out.args.aux = out.aux;
  for (int a : folds) if (m.nodes[a].flags & FC_NODE_SINGLE_PASS) out.args.flags |= kSinglePass;
  for (int a : foldsegs) if (m.nodes[a].flags & FC_NODE_SINGLE_PASS) out.args.flags |= kSinglePass;
  for (int k = 0; k < kMaxOut; ++k)
    if (out.out_nodes[k] >= 0 && !m.out_edges[out.out_nodes[k]].empty()) out.args.flags |= kKeepOut << k;
  out.externals = b.externals;
  const Instance *inst = find_instance(sig, out.args);
  if (!inst && !any.empty() && b.code_ok && b.on_stack == 0) inst = find_instance(any, out.args);
  if (!inst && interpretable) inst = interpreter_instance();
  if (!inst) return unsupported("no kernel instance for cluster " + sig);
  out.instance = inst;
  return FC_OK;
}

std::vector<std::vector<int>> clusters_of(const Model &m, const Clustering &c) {
  std::map<int, std::vector<int>> by_pi;
  for (int a = 0; a < m.n; ++a) if (!m.is_input(a)) by_pi[c.pi[a]].push_back(a);
  std::vector<std::vector<int>> r;
  for (auto &kv : by_pi) r.push_back(kv.second);
  return r;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// the clusters run one after the other, so they share one workspace: the largest any of them asks for
static size_t workspace_bytes_for(const Model &m, const Clustering &c) {
  size_t most = 0;
  for (const auto &members : clusters_of(m, c)) {
    ClusterLaunch cl;
    std::string err;
    if (plan_cluster(m, c, members, cl, err) != FC_OK || cl.kind != ClusterLaunch::Kernel || !cl.instance->workspace) continue;
    most = std::max(most, cl.instance->workspace(cl.args));
  }
  return most;
}

size_t scratch_bytes_for(const Model &m, const Clustering &c) {
  size_t total = FC_SCRATCH_CONTROL_BYTES;
  for (int a = 0; a < m.n; ++a)
    if (!m.is_input(a) && !c.fused_away[a] && m.nodes[a].kind != FC_SCATTER && m.nodes[a].kind != FC_FORCE)
      total += align_up(std::max<size_t>((size_t)m.bytes(a), 4), 256);
  return total + align_up(workspace_bytes_for(m, c), 256);
}

int prepare_run(PreparedRun &r, std::string &err) {
  // plan every cluster before the first launch, so that an unsupported cluster
  // leaves no partial results behind
  r.launches.clear();
  for (const auto &members : clusters_of(r.model, r.clustering)) {
    ClusterLaunch cl;
    int rc = plan_cluster(r.model, r.clustering, members, cl, err);
    if (rc != FC_OK) return rc;
    r.launches.push_back(cl);
  }
  return FC_OK;
}

int run_prepared(const PreparedRun &r, const fc_buffer *bufs, void *scratch, size_t scratch_bytes, hipStream_t stream,
                 std::string &err) {
  const Model &m = r.model;
  const Clustering &c = r.clustering;
  if (!bufs) { err = "null buffer table"; return FC_E_ARG; }
  if (!scratch || ((uintptr_t)scratch & 255u) || scratch_bytes < FC_SCRATCH_CONTROL_BYTES) {
    err = "scratch must be 256-byte aligned and at least FC_SCRATCH_CONTROL_BYTES";
    return FC_E_SCRATCH;
  }
  // resolve the device buffer of every array that reaches memory
  std::vector<void *> ptr(m.n, nullptr);
  size_t cursor = FC_SCRATCH_CONTROL_BYTES;
  for (int a = 0; a < m.n; ++a) {
    const fc_node &nd = m.nodes[a];
    const size_t need = std::max<size_t>((size_t)m.bytes(a), nd.kind == FC_FOLD ? 4 : 0);
    if (nd.kind == FC_SCATTER) {
      ptr[a] = ptr[nd.arg[0]];
      if (bufs[a].ptr && bufs[a].ptr != ptr[a]) { err = "scatter " + std::to_string(a) + " must share the buffer of its destination"; return FC_E_UNBOUND; }
      continue;
    }
    if (!m.is_input(a) && c.fused_away[a]) continue;
    if (bufs[a].ptr) {
      if ((size_t)bufs[a].bytes < need) { err = "buffer of node " + std::to_string(a) + " is too small"; return FC_E_UNBOUND; }
      if ((uintptr_t)bufs[a].ptr & 15u) { err = "buffer of node " + std::to_string(a) + " is not 16-byte aligned"; return FC_E_UNBOUND; }
      ptr[a] = bufs[a].ptr;
    } else if (m.is_input(a)) {
      if (need == 0) { ptr[a] = scratch; continue; }   // empty array: any valid pointer
      err = "input " + std::to_string(a) + " is not bound";
      return FC_E_UNBOUND;
    } else if (nd.kind == FC_FORCE) {
      ptr[a] = ptr[nd.arg[0]];
    } else {
      size_t sz = align_up(std::max<size_t>(need, 4), 256);
      if (cursor + sz > scratch_bytes) { err = "scratch too small for the manifest intermediates"; return FC_E_SCRATCH; }
      ptr[a] = static_cast<char *>(scratch) + cursor;
      cursor += sz;
    }
  }
  LaunchCtx ctx;
  ctx.stream = stream;
  ctx.ctl = static_cast<Control *>(scratch);
  ctx.partials = reinterpret_cast<unsigned long long *>(static_cast<char *>(scratch) + kPartialsOffset);
  ctx.status = reinterpret_cast<unsigned long long *>(static_cast<char *>(scratch) + kStatusOffset);
  ctx.max_tiles = kMaxTiles;
  // what is left of scratch after the intermediates is the clusters' common workspace
  const size_t workspace_at = align_up(cursor, 256);

  for (ClusterLaunch cl : r.launches) {
    if (cl.kind == ClusterLaunch::Alias) {
      if (bufs[cl.alias_node].ptr && bufs[cl.alias_node].ptr != ptr[cl.alias_of]) {
        hipError_t e = hipMemcpyAsync(bufs[cl.alias_node].ptr, ptr[cl.alias_of], (size_t)m.bytes(cl.alias_node),
                                      hipMemcpyDeviceToDevice, stream);
        if (e != hipSuccess) { err = hipGetErrorString(e); return FC_E_HIP; }
      }
      continue;
    }
    for (size_t k = 0; k < cl.externals.size(); ++k) {
      cl.args.in[k] = ptr[cl.externals[k]];
      if (!cl.args.in[k]) { err = "array " + std::to_string(cl.externals[k]) + " read before it exists"; return FC_E_UNBOUND; }
    }
    if (cl.offsets_node >= 0) cl.args.in[kMaxIn - 1] = ptr[cl.offsets_node];
    for (int k = 0; k < kMaxOut; ++k)
      if (cl.out_nodes[k] >= 0) {
        cl.args.out[k] = ptr[cl.out_nodes[k]];
        if (!cl.args.out[k]) { err = "array " + std::to_string(cl.out_nodes[k]) + " has no buffer"; return FC_E_UNBOUND; }
      }
    ctx.workspace = nullptr;
    if (cl.instance->workspace) {
      const size_t need = cl.instance->workspace(cl.args);
      if (workspace_at + need > scratch_bytes) { err = "scratch too small for the workspace of " + cl.sig; return FC_E_SCRATCH; }
      ctx.workspace = static_cast<char *>(scratch) + workspace_at;
    }
    hipError_t e = cl.instance->launch(cl.args, ctx);
    if (e != hipSuccess) {
      int count = -1, dev = -1;
      hipError_t e2 = hipGetDeviceCount(&count);
      hipError_t e3 = hipGetDevice(&dev);
      err = std::string("launch of ") + cl.sig + ": " + hipGetErrorString(e) + " (devices visible to the library: " +
            std::to_string(count) + ", current " + std::to_string(dev) + ", status " + std::to_string((int)e2) + "/" +
            std::to_string((int)e3) + ")";
      return FC_E_HIP;
    }
  }
  return FC_OK;
}

}  // namespace fc
