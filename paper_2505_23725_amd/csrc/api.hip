// C-ABI entry points, host-side argument validation, launch planning and the optional
// timing recorder.  Nothing here allocates device memory or synchronises the stream.
#include <atomic>
#include <cmath>
#include <mutex>
#include <vector>

#include "common.h"

// Work space of newton_schulz_static_scratch.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address differs per GPU and is looked up once per device.
static __device__ __align__(256) unsigned char scratch[MLC_STATIC_SCRATCH_BYTES];

namespace mlc {

// ---- timing recorder -------------------------------------------------------------
namespace {
struct TimingRecord { int family; hipEvent_t start, stop; double flops, bytes; };
struct TimingState {
  std::mutex mu;
  std::atomic<bool> enabled{false};   // read on every launch without taking the lock
  std::vector<TimingRecord> records;
  std::vector<hipEvent_t> pool;
};
TimingState& timing() { static TimingState s; return s; }
constexpr size_t kMaxRecords = 1u << 18;

hipEvent_t get_event(TimingState& t) {
  if (!t.pool.empty()) { hipEvent_t e = t.pool.back(); t.pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

LaunchScope::LaunchScope(int family, hipStream_t s, double flops, double bytes) : slot(-1), stream(s) {
  TimingState& t = timing();
  if (!t.enabled.load(std::memory_order_relaxed)) return;
  std::lock_guard<std::mutex> lock(t.mu);
  if (t.records.size() >= kMaxRecords) return;
  TimingRecord r{family, get_event(t), get_event(t), flops, bytes};
  if (!r.start || !r.stop) {          // keep whichever of the two was created
    if (r.start) t.pool.push_back(r.start);
    if (r.stop) t.pool.push_back(r.stop);
    return;
  }
  (void)hipEventRecord(r.start, stream);
  t.records.push_back(r);
  slot = (int)t.records.size() - 1;
}
LaunchScope::~LaunchScope() {
  if (slot < 0) return;
  TimingState& t = timing();
  std::lock_guard<std::mutex> lock(t.mu);
  if (slot < (int)t.records.size()) (void)hipEventRecord(t.records[slot].stop, stream);
}

namespace {

constexpr int64_t PAD = 128;               // GEMM tile granularity of the work-space layout
// Row pitch of every work-space matrix = padded row length + 64 elements (one 128-byte
// line): a pitch with a large power-of-two factor (5120 B, 6144 B, 10240 B ...) makes the
// rows a workgroup fetches together fall on few L2 channels.
constexpr int64_t PITCH_SKEW = 64;
constexpr int64_t WS_ALIGN = 256;
constexpr int MAX_NBLK = 1024;             // workgroups per matrix in the norm reduction
constexpr int64_t MAX_CHUNK = 65535;       // gridDim.y limit

bool valid_dtype(int d) { return d == MLC_F32 || d == MLC_BF16; }

int check_shape(int64_t count, int64_t m, int64_t n) {
  if (count < 1 || m < 1 || n < 1) return MLC_ERR_SHAPE;
  const int64_t lim = (int64_t)1 << 30;    // per-dimension limit keeps int indexing valid
  if (m > lim || n > lim || count > lim) return MLC_ERR_SHAPE;
  const int64_t mp = round_up(m, PAD), np = round_up(n, PAD);
  if (mp > ((int64_t)1 << 31) / (np + PITCH_SKEW)) {   // one padded matrix must stay below 2^31 elements
    return MLC_ERR_SHAPE;
  }
  if ((double)count * (double)mp * (double)np >= 4.0e18) return MLC_ERR_SHAPE;
  return MLC_OK;
}

// Work-space layout for a chunk of c matrices:  X0 | X1 | A | B | scale | partials
struct NsPlan {
  int64_t m, n, mp, np, sp;
  int64_t ldx, lds;        // row pitch (elements) of X0/X1 and of A/B
  int nblk;
  size_t per_matrix;       // bytes that scale with the chunk size
  size_t x_bytes, s_bytes; // per matrix
};

NsPlan make_plan(int64_t m, int64_t n) {
  NsPlan p;
  p.m = m; p.n = n;
  p.mp = round_up(m, PAD); p.np = round_up(n, PAD);
  p.sp = p.mp < p.np ? p.mp : p.np;
  p.ldx = p.np + PITCH_SKEW; p.lds = p.sp + PITCH_SKEW;
  const int64_t items = p.mp * (p.np / 8);
  int64_t nblk = items / (256 * 4);
  if (nblk < 1) nblk = 1;
  if (nblk > MAX_NBLK) nblk = MAX_NBLK;
  p.nblk = (int)nblk;
  p.x_bytes = (size_t)p.mp * p.ldx * 2;
  p.s_bytes = (size_t)p.sp * p.lds * 2;
  p.per_matrix = 2 * p.x_bytes + 2 * p.s_bytes + (size_t)WS_ALIGN /*scale slot*/ +
                 (size_t)round_up((int64_t)p.nblk * 4, WS_ALIGN);
  return p;
}

struct NsBuffers { bf16_t* X[2]; bf16_t* A; bf16_t* B; float* scale; float* partials; };

NsBuffers carve(const NsPlan& p, void* ws, int64_t chunk) {
  unsigned char* base = (unsigned char*)ws;
  NsBuffers b;
  b.X[0] = (bf16_t*)base; base += p.x_bytes * chunk;
  b.X[1] = (bf16_t*)base; base += p.x_bytes * chunk;
  b.A = (bf16_t*)base; base += p.s_bytes * chunk;
  b.B = (bf16_t*)base; base += p.s_bytes * chunk;
  b.scale = (float*)base; base += (size_t)WS_ALIGN * chunk;
  b.partials = (float*)base;
  return b;
}

int64_t chunk_for(const NsPlan& p, size_t ws_bytes, int64_t count) {
  int64_t c = (int64_t)(ws_bytes / p.per_matrix);
  if (c > count) c = count;
  if (c > MAX_CHUNK) c = MAX_CHUNK;
  return c;
}

// One batch of same-shape matrices on its way through Newton-Schulz: its (unnormalised) input
// sits in w.X[0], the per-matrix partial sums of squares in w.partials.
// With fuse_W set, the last product of the last iteration writes the parameter update itself,
// W <- fuse_decay * W - fuse_step * O (paper Sec. 2 "Muon"), instead of storing O: O is then
// never rounded to bf16 nor read back, and result_buf is -1 on return.
struct NsJob {
  NsPlan p; NsBuffers w; int64_t chunk; int result_buf;
  bf16_t* fuse_W = nullptr; float fuse_decay = 0.f, fuse_step = 0.f;
};
// The update can ride on the last product when W is bf16 and has the shape the products work
// on (no padding), and the matrices are not small enough for the one-launch chain.
static bool can_fuse_update(const NsPlan& p, int param_dtype, int iters) {
  return iters >= 1 && param_dtype == MLC_BF16 && p.m == p.mp && p.n == p.np && !ns_chain_small_fits(p.mp, p.np);
}
constexpr int MAX_NS_JOBS = 16;

// The three products of one iteration of job j (X = current buffer, Xn = the other one).
//
// The polynomial is folded before the last product: B' = a I + b A + c A^2, X <- B' X,
// which is the printed iteration with one rounding to bf16 fewer.  The normalisation is
// folded into the first iteration's scalars: A_0 = s^2 U U^T, X_1 = s B' U.
static GemmDesc gram_desc(const NsJob& j, const bf16_t* X, bool first) {
  const NsPlan& p = j.p;
  const bool wide = p.mp <= p.np;
  const int64_t xs = p.mp * p.ldx, ss = p.sp * p.lds;
  GemmDesc g{};
  // Gram matrix: A = X X^T (wide) or X^T X (tall)
  g.A = X; g.lda = p.ldx; g.strideA = xs; g.a_kstrided = wide ? 0 : 1;
  g.B = X; g.ldb = p.ldx; g.strideB = xs; g.b_kstrided = wide ? 0 : 1;
  g.D = j.w.A; g.ldd = p.lds; g.strideD = ss;
  g.C = nullptr;
  g.M = (int)p.sp; g.N = (int)p.sp; g.K = (int)(wide ? p.np : p.mp); g.batch = (int)j.chunk;
  g.alpha = 1.f; g.beta = 0.f; g.gamma = 0.f;
  g.bscale = first ? j.w.scale : nullptr; g.bscale_pow = 2;
  g.symmetric = 1;     // only the lower triangle of tiles is computed, then mirrored
  return g;
}
static GemmDesc poly_desc(const NsJob& j, float a, float b, float c) {
  const NsPlan& p = j.p;
  const int64_t ss = p.sp * p.lds;
  // Polynomial: B' = c A A + b A + a I.  A is symmetric, so either operand may be read
  // along rows or along columns; the K-contiguous LDS path is the faster one.
  GemmDesc g{};
  g.A = j.w.A; g.lda = p.lds; g.strideA = ss; g.a_kstrided = 0;
  g.B = j.w.A; g.ldb = p.lds; g.strideB = ss; g.b_kstrided = 0;
  g.D = j.w.B; g.ldd = p.lds; g.strideD = ss;
  g.C = j.w.A; g.ldc = p.lds; g.strideC = ss;
  g.M = g.N = g.K = (int)p.sp; g.batch = (int)j.chunk;
  g.alpha = c; g.beta = b; g.gamma = a;
  g.symmetric = 1;
  return g;
}
static GemmDesc apply_desc(const NsJob& j, const bf16_t* X, bf16_t* Xn, bool first) {
  const NsPlan& p = j.p;
  const bool wide = p.mp <= p.np;
  const int64_t xs = p.mp * p.ldx, ss = p.sp * p.lds;
  // Apply: X <- B' X (wide) or X B' (tall; B' symmetric)
  GemmDesc g{};
  if (wide) {     // B' symmetric: read along rows (K-contiguous); X has k as its slow index
    g.A = j.w.B; g.lda = p.lds; g.strideA = ss; g.a_kstrided = 0;
    g.B = X; g.ldb = p.ldx; g.strideB = xs; g.b_kstrided = 1;
    g.M = (int)p.mp; g.N = (int)p.np; g.K = (int)p.mp;
  } else {
    g.A = X; g.lda = p.ldx; g.strideA = xs; g.a_kstrided = 0;
    g.B = j.w.B; g.ldb = p.lds; g.strideB = ss; g.b_kstrided = 0;
    g.M = (int)p.mp; g.N = (int)p.np; g.K = (int)p.np;
  }
  g.D = Xn; g.ldd = p.ldx; g.strideD = xs;
  g.C = nullptr; g.batch = (int)j.chunk;
  g.alpha = 1.f; g.beta = 0.f; g.gamma = 0.f;
  g.bscale = first ? j.w.scale : nullptr; g.bscale_pow = 1;
  return g;
}
// The same product with the parameter update as its epilogue: D = decay * W - step * (B' X).
static GemmDesc apply_update_desc(const NsJob& j, const bf16_t* X, bool first) {
  GemmDesc g = apply_desc(j, X, j.fuse_W, first);
  g.ldd = j.p.n; g.strideD = j.p.m * j.p.n;
  g.C = j.fuse_W; g.ldc = g.ldd; g.strideC = g.strideD;
  g.alpha = -j.fuse_step; g.beta = j.fuse_decay;
  return g;
}

// The `iters` Newton-Schulz iterations on n independent jobs.  On return result_buf of a job
// is the index of the buffer that holds its result; with iters == 0 the result is X[0] still
// unscaled, and its factor 1/(norm+eps) sits in `scale`.  The same product of several jobs
// goes out as one set, so that products of equal depth can share launches.
int run_ns_jobs(NsJob* jobs, int n, int iters, float a, float b, float c, float eps, hipStream_t stream) {
  if (n < 1 || n > MAX_NS_JOBS) return MLC_ERR_ARG;
  NsJob* big[MAX_NS_JOBS];
  int nbig = 0;
  for (int i = 0; i < n; ++i) {
    NsJob& j = jobs[i];
    if (iters >= 1 && ns_chain_small_fits(j.p.mp, j.p.np)) {
      // small matrices: norm and all iterations in one launch, X and A resident in LDS
      j.result_buf = 1;
      const int rc = launch_ns_chain_small(j.w.X[0], j.w.X[1], j.p.ldx, j.p.mp * j.p.ldx, j.p.mp, j.p.np,
                                           j.w.partials, j.p.nblk, eps, j.chunk, iters, a, b, c, stream);
      if (rc != MLC_OK) return rc;
      continue;
    }
    const int rc = launch_norm_finalize(j.w.partials, j.p.nblk, j.w.scale, j.chunk, eps, stream);
    if (rc != MLC_OK) return rc;
    j.result_buf = 0;
    big[nbig++] = &j;
  }
  GemmDesc d[MAX_NS_JOBS];
  int cur = 0;
  for (int it = 0; it < iters && nbig > 0; ++it) {
    for (int i = 0; i < nbig; ++i) d[i] = gram_desc(*big[i], big[i]->w.X[cur], it == 0);
    int rc = launch_ns_gemm_set(d, nbig, stream);
    if (rc != MLC_OK) return rc;
    for (int i = 0; i < nbig; ++i) d[i] = poly_desc(*big[i], a, b, c);
    rc = launch_ns_gemm_set(d, nbig, stream);
    if (rc != MLC_OK) return rc;
    const bool last = it + 1 == iters;
    for (int i = 0; i < nbig; ++i)
      d[i] = (last && big[i]->fuse_W) ? apply_update_desc(*big[i], big[i]->w.X[cur], it == 0)
                                      : apply_desc(*big[i], big[i]->w.X[cur], big[i]->w.X[cur ^ 1], it == 0);
    rc = launch_ns_gemm_set(d, nbig, stream);
    if (rc != MLC_OK) return rc;
    cur ^= 1;
  }
  for (int i = 0; i < nbig; ++i) big[i]->result_buf = (iters >= 1 && big[i]->fuse_W) ? -1 : cur;
  return MLC_OK;
}

int run_ns_chunk(const NsPlan& p, const NsBuffers& w, int64_t chunk, int iters, float a, float b,
                 float c, float eps, hipStream_t stream, int* result_buf, bf16_t* fuse_W = nullptr,
                 float fuse_decay = 0.f, float fuse_step = 0.f) {
  NsJob j{p, w, chunk, 0};
  j.fuse_W = fuse_W; j.fuse_decay = fuse_decay; j.fuse_step = fuse_step;
  const int rc = run_ns_jobs(&j, 1, iters, a, b, c, eps, stream);
  *result_buf = j.result_buf;
  return rc;
}

int check_workspace(const void* ws, size_t bytes, size_t need) {
  if (!ws) return MLC_ERR_WORKSPACE;
  if (((uintptr_t)ws) % WS_ALIGN) return MLC_ERR_WORKSPACE;
  if (bytes < need) return MLC_ERR_WORKSPACE;
  return MLC_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p) % 16 == 0; }

size_t elem_size(int dtype) { return dtype == MLC_F32 ? 4 : 2; }

}  // namespace
}  // namespace mlc

using namespace mlc;

extern "C" {

const char* muloco_strerror(int code) {
  switch (code) {
    case MLC_OK: return "ok";
    case MLC_ERR_NULL: return "null pointer";
    case MLC_ERR_SHAPE: return "bad shape";
    case MLC_ERR_DTYPE: return "bad dtype";
    case MLC_ERR_WORKSPACE: return "workspace null, misaligned or too small";
    case MLC_ERR_ARG: return "argument out of range";
    case MLC_ERR_LAUNCH: return "kernel launch failed";
    case MLC_ERR_UNSUPPORTED: return "unsupported combination";
    case MLC_ERR_SCRATCH: return "one matrix of this shape does not fit the built-in scratch buffer";
    default: return "unknown error";
  }
}

size_t newton_schulz_workspace_min_bytes(int64_t m, int64_t n) {
  if (check_shape(1, m, n) != MLC_OK) return 0;
  return make_plan(m, n).per_matrix;
}

size_t newton_schulz_workspace_bytes(int64_t count, int64_t m, int64_t n) {
  if (check_shape(count, m, n) != MLC_OK) return 0;
  const int64_t c = count > MAX_CHUNK ? MAX_CHUNK : count;
  return make_plan(m, n).per_matrix * (size_t)c;
}

// Shared body of newton_schulz and newton_schulz_static_scratch; `need_error` is the code
// returned when the work space cannot hold one matrix.
static int newton_schulz_in(const void* in, void* out, int io_dtype, int64_t count, int64_t m, int64_t n,
                            int iters, float a, float b, float c, float eps, void* workspace,
                            size_t workspace_bytes, int need_error, hipStream_t stream) {
  const NsPlan p = make_plan(m, n);
  if (workspace_bytes < p.per_matrix) return need_error;
  int rc = check_workspace(workspace, workspace_bytes, p.per_matrix);
  if (rc != MLC_OK) return rc;
  const int64_t chunk = chunk_for(p, workspace_bytes, count);
  const size_t es = elem_size(io_dtype);
  for (int64_t c0 = 0; c0 < count; c0 += chunk) {
    const int64_t cc = count - c0 < chunk ? count - c0 : chunk;
    const NsBuffers w = carve(p, workspace, chunk);
    const unsigned char* src = (const unsigned char*)in + (size_t)c0 * m * n * es;
    unsigned char* dst = (unsigned char*)out + (size_t)c0 * m * n * es;
    rc = launch_ns_load(src, io_dtype, w.X[0], w.partials, p.nblk, cc, m, n, p.mp, p.np, p.ldx, stream);
    if (rc != MLC_OK) return rc;
    int res = 0;
    rc = run_ns_chunk(p, w, cc, iters, a, b, c, eps, stream, &res);
    if (rc != MLC_OK) return rc;
    rc = launch_ns_store(w.X[res], iters == 0 ? w.scale : nullptr, dst, io_dtype, cc, m, n, p.mp,
                         p.ldx, stream);
    if (rc != MLC_OK) return rc;
  }
  return MLC_OK;
}

static int check_ns_args(const void* in, const void* out, int io_dtype, int64_t count, int64_t m,
                         int64_t n, int iters, float eps) {
  if (!in || !out) return MLC_ERR_NULL;
  if (!valid_dtype(io_dtype)) return MLC_ERR_DTYPE;
  const int rc = check_shape(count, m, n);
  if (rc != MLC_OK) return rc;
  if (iters < 0 || !(eps >= 0.f)) return MLC_ERR_ARG;
  if (!aligned16(in) || !aligned16(out)) return MLC_ERR_ARG;
  return MLC_OK;
}

int newton_schulz(const void* in, void* out, int io_dtype, int64_t count, int64_t m, int64_t n,
                  int iters, float a, float b, float c, float eps, void* workspace,
                  size_t workspace_bytes, void* stream_) {
  const int rc = check_ns_args(in, out, io_dtype, count, m, n, iters, eps);
  if (rc != MLC_OK) return rc;
  if (!workspace) return MLC_ERR_WORKSPACE;
  return newton_schulz_in(in, out, io_dtype, count, m, n, iters, a, b, c, eps, workspace, workspace_bytes,
                          MLC_ERR_WORKSPACE, (hipStream_t)stream_);
}

// Device address of `scratch` on the current device, looked up on the first call there.
static int static_scratch_address(void** out) {
  static std::atomic<void*> address[MAX_DEVICES];
  const int slot = device_slot();
  if (slot < 0) return MLC_ERR_UNSUPPORTED;
  void* p = address[slot].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MLC_ERR_LAUNCH;
    address[slot].store(p, std::memory_order_release);   // two threads racing store the same value
  }
  *out = p;
  return MLC_OK;
}

int newton_schulz_static_scratch(const void* in, void* out, int io_dtype, int64_t count, int64_t m,
                                 int64_t n, int iters, float a, float b, float c, float eps,
                                 void* stream_) {
  int rc = check_ns_args(in, out, io_dtype, count, m, n, iters, eps);
  if (rc != MLC_OK) return rc;
  if (make_plan(m, n).per_matrix > MLC_STATIC_SCRATCH_BYTES) return MLC_ERR_SCRATCH;
  void* ws = nullptr;
  rc = static_scratch_address(&ws);
  if (rc != MLC_OK) return rc;
  return newton_schulz_in(in, out, io_dtype, count, m, n, iters, a, b, c, eps, ws, MLC_STATIC_SCRATCH_BYTES,
                          MLC_ERR_SCRATCH, (hipStream_t)stream_);
}

static int check_inner_groups(const mlc_inner_group* groups, int n_groups) {
  if (!groups) return MLC_ERR_NULL;
  if (n_groups < 0) return MLC_ERR_ARG;
  for (int i = 0; i < n_groups; ++i) {
    const mlc_inner_group& g = groups[i];
    if (!g.param || !g.grad || !g.momentum) return MLC_ERR_NULL;
    if (!valid_dtype(g.param_dtype) || !valid_dtype(g.grad_dtype)) return MLC_ERR_DTYPE;
    const int rc = check_shape(g.count, g.m, g.n);
    if (rc != MLC_OK) return rc;
    if (!aligned16(g.param) || !aligned16(g.grad) || !aligned16(g.momentum)) return MLC_ERR_ARG;
  }
  return MLC_OK;
}

// Work space with which all groups are resident at once, each as a single batch: the sum over
// groups (0 when a group is too large to be one batch).
static size_t inner_workspace_all(const mlc_inner_group* groups, int n_groups) {
  size_t need = 0;
  for (int i = 0; i < n_groups; ++i) {
    if (groups[i].count > MAX_CHUNK) return 0;
    need += make_plan(groups[i].m, groups[i].n).per_matrix * (size_t)groups[i].count;
  }
  return need;
}

size_t muloco_inner_workspace_bytes(const mlc_inner_group* groups, int n_groups) {
  if (check_inner_groups(groups, n_groups) != MLC_OK) return 0;
  const size_t all = (n_groups <= MAX_NS_JOBS) ? inner_workspace_all(groups, n_groups) : 0;
  if (all) return all;
  size_t need = 0;
  for (int i = 0; i < n_groups; ++i) {
    const size_t b = newton_schulz_workspace_bytes(groups[i].count, groups[i].m, groups[i].n);
    if (b > need) need = b;
  }
  return need;
}

size_t muloco_inner_workspace_min_bytes(const mlc_inner_group* groups, int n_groups) {
  if (check_inner_groups(groups, n_groups) != MLC_OK) return 0;
  size_t need = 0;
  for (int i = 0; i < n_groups; ++i) {
    const size_t b = newton_schulz_workspace_min_bytes(groups[i].m, groups[i].n);
    if (b > need) need = b;
  }
  return need;
}

int muloco_inner_step(const mlc_inner_group* groups, int n_groups, const mlc_muon_hparams* hp,
                      void* workspace, size_t workspace_bytes, void* stream_) {
  if (!hp) return MLC_ERR_NULL;
  int rc = check_inner_groups(groups, n_groups);
  if (rc != MLC_OK) return rc;
  if (hp->ns_iters < 0 || !(hp->ns_eps >= 0.f)) return MLC_ERR_ARG;
  if (n_groups == 0) return MLC_OK;
  rc = check_workspace(workspace, workspace_bytes, muloco_inner_workspace_min_bytes(groups, n_groups));
  if (rc != MLC_OK) return rc;
  hipStream_t stream = (hipStream_t)stream_;
  const float decay_factor = 1.0f - hp->eta * hp->weight_decay;
  // With room for every group at once the groups go through Newton-Schulz side by side, so that
  // their products of equal depth share launches; otherwise one group after the other, in
  // chunks that fit.  Both give the same bits.
  const size_t all = (n_groups >= 2 && n_groups <= MAX_NS_JOBS) ? inner_workspace_all(groups, n_groups) : 0;
  if (all && workspace_bytes >= all) {
    NsJob jobs[MAX_NS_JOBS];
    unsigned char* base = (unsigned char*)workspace;
    for (int gi = 0; gi < n_groups; ++gi) {
      const mlc_inner_group& g = groups[gi];
      jobs[gi].p = make_plan(g.m, g.n);
      jobs[gi].chunk = g.count;
      jobs[gi].w = carve(jobs[gi].p, base, g.count);
      jobs[gi].result_buf = 0;
      if (can_fuse_update(jobs[gi].p, g.param_dtype, hp->ns_iters)) {
        jobs[gi].fuse_W = (bf16_t*)g.param;
        jobs[gi].fuse_decay = decay_factor;
        jobs[gi].fuse_step = hp->eta * g.lr_scale;
      }
      base += jobs[gi].p.per_matrix * (size_t)g.count;
      rc = launch_momentum(g.grad, g.grad_dtype, g.momentum, jobs[gi].w.X[0], jobs[gi].w.partials,
                           jobs[gi].p.nblk, g.count, g.m, g.n, jobs[gi].p.mp, jobs[gi].p.np, jobs[gi].p.ldx,
                           hp->beta, hp->nesterov, stream);
      if (rc != MLC_OK) return rc;
    }
    rc = run_ns_jobs(jobs, n_groups, hp->ns_iters, hp->ns_a, hp->ns_b, hp->ns_c, hp->ns_eps, stream);
    if (rc != MLC_OK) return rc;
    for (int gi = 0; gi < n_groups; ++gi) {
      const mlc_inner_group& g = groups[gi];
      const NsJob& j = jobs[gi];
      if (j.result_buf < 0) continue;      // the last product wrote W
      rc = launch_param_update(g.param, g.param_dtype, j.w.X[j.result_buf],
                               hp->ns_iters == 0 ? j.w.scale : nullptr, g.count, g.m, g.n, j.p.mp, j.p.ldx,
                               decay_factor, hp->eta * g.lr_scale, stream);
      if (rc != MLC_OK) return rc;
    }
    return MLC_OK;
  }
  for (int gi = 0; gi < n_groups; ++gi) {
    const mlc_inner_group& g = groups[gi];
    const NsPlan p = make_plan(g.m, g.n);
    const int64_t chunk = chunk_for(p, workspace_bytes, g.count);
    const size_t mat = (size_t)g.m * g.n;
    for (int64_t c0 = 0; c0 < g.count; c0 += chunk) {
      const int64_t cc = g.count - c0 < chunk ? g.count - c0 : chunk;
      const NsBuffers w = carve(p, workspace, chunk);
      const unsigned char* grad = (const unsigned char*)g.grad + c0 * mat * elem_size(g.grad_dtype);
      unsigned char* param = (unsigned char*)g.param + c0 * mat * elem_size(g.param_dtype);
      float* mom = g.momentum + c0 * mat;
      rc = launch_momentum(grad, g.grad_dtype, mom, w.X[0], w.partials, p.nblk, cc, g.m, g.n, p.mp,
                           p.np, p.ldx, hp->beta, hp->nesterov, stream);
      if (rc != MLC_OK) return rc;
      int res = 0;
      const bool fuse = can_fuse_update(p, g.param_dtype, hp->ns_iters);
      rc = run_ns_chunk(p, w, cc, hp->ns_iters, hp->ns_a, hp->ns_b, hp->ns_c, hp->ns_eps, stream, &res,
                        fuse ? (bf16_t*)param : nullptr, decay_factor, hp->eta * g.lr_scale);
      if (rc != MLC_OK) return rc;
      if (res < 0) continue;               // the last product wrote W
      rc = launch_param_update(param, g.param_dtype, w.X[res], hp->ns_iters == 0 ? w.scale : nullptr,
                               cc, g.m, g.n, p.mp, p.ldx, decay_factor, hp->eta * g.lr_scale, stream);
      if (rc != MLC_OK) return rc;
    }
  }
  return MLC_OK;
}

static int check_outer(const mlc_outer_group* groups, int n_groups, const mlc_outer_hparams* hp,
                       bool need_update_state, bool topk = false) {
  if (!hp || !groups) return MLC_ERR_NULL;
  if (n_groups < 0) return MLC_ERR_ARG;
  if (hp->K < 1 || hp->K > MLC_MAX_WORKERS) return MLC_ERR_ARG;
  if (hp->quant_bits != 0 && hp->quant_bits != 2 && hp->quant_bits != 4 && hp->quant_bits != 8)
    return MLC_ERR_ARG;
  if (hp->error_feedback != 0 && hp->error_feedback != 1) return MLC_ERR_ARG;
  if (topk && hp->quant_bits != 0) return MLC_ERR_ARG;
  if (hp->error_feedback && ((hp->quant_bits == 0 && !topk) || !(hp->ef_beta >= 0.f))) return MLC_ERR_ARG;
  if (hp->second_quantisation != 0 && hp->second_quantisation != 1) return MLC_ERR_ARG;
  if (hp->second_quantisation && hp->quant_bits == 0) return MLC_ERR_ARG;
  if ((hp->quant_offset != 0 && hp->quant_offset != 1) ||
      (hp->quant_per_matrix != 0 && hp->quant_per_matrix != 1))
    return MLC_ERR_ARG;
  if ((hp->quant_offset || hp->quant_per_matrix) && hp->quant_bits == 0) return MLC_ERR_ARG;
  if (hp->second_quantisation && hp->quant_per_matrix) return MLC_ERR_UNSUPPORTED;
  for (int i = 0; i < n_groups; ++i) {
    const mlc_outer_group& g = groups[i];
    if (!g.worker_params || !g.global_param) return MLC_ERR_NULL;
    if (need_update_state && !g.outer_momentum) return MLC_ERR_NULL;
    if (!valid_dtype(g.worker_dtype) || !valid_dtype(g.global_dtype)) return MLC_ERR_DTYPE;
    const int rc = check_shape(g.count, g.m, g.n);
    if (rc != MLC_OK) return rc;
    if (!aligned16(g.global_param) || (g.outer_momentum && !aligned16(g.outer_momentum)))
      return MLC_ERR_ARG;
    for (int k = 0; k < hp->K; ++k) {
      if (!g.worker_params[k]) return MLC_ERR_NULL;
      if (!aligned16(g.worker_params[k])) return MLC_ERR_ARG;
    }
    if (hp->quant_bits) {
      if (g.n % (8 / hp->quant_bits)) return MLC_ERR_SHAPE;
      if (!g.codes || !g.scales) return MLC_ERR_NULL;
      for (int k = 0; k < hp->K; ++k) {
        if (!g.codes[k] || !g.scales[k]) return MLC_ERR_NULL;
        if (!aligned16(g.codes[k]) || !aligned16(g.scales[k])) return MLC_ERR_ARG;
      }
    }
    if (hp->quant_offset) {
      if (!g.offsets) return MLC_ERR_NULL;
      for (int k = 0; k < hp->K; ++k) {
        if (!g.offsets[k]) return MLC_ERR_NULL;
        if (!aligned16(g.offsets[k])) return MLC_ERR_ARG;
      }
    }
    if (hp->quant_per_matrix && g.count > 65535) return MLC_ERR_SHAPE;
    if (hp->second_quantisation) {
      if ((g.mean_codes && !aligned16(g.mean_codes)) || (g.mean_scales && !aligned16(g.mean_scales)) ||
          (g.mean_offsets && !aligned16(g.mean_offsets)))
        return MLC_ERR_ARG;
      if (g.n % 8 || g.n > 24576 || (g.worker_dtype == MLC_F32 && g.global_dtype == MLC_BF16))
        return MLC_ERR_UNSUPPORTED;
    }
    if (hp->error_feedback) {
      if (!g.residuals) return MLC_ERR_NULL;
      for (int k = 0; k < hp->K; ++k) {
        if (!g.residuals[k]) return MLC_ERR_NULL;
        if (!aligned16(g.residuals[k])) return MLC_ERR_ARG;
      }
    }
  }
  return MLC_OK;
}

struct OuterPtrs { WorkerPtrs w; CodePtrs c; ScalePtrs s; OffsetPtrs o; ResidualPtrs e; };

static void gather_ptrs(const mlc_outer_group& g, const mlc_outer_hparams& hp, OuterPtrs& p) {
  const int K = hp.K;
  const bool quant = hp.quant_bits != 0;
  for (int k = 0; k < MLC_MAX_WORKERS; ++k) {
    p.w.p[k] = k < K ? g.worker_params[k] : nullptr;
    p.c.p[k] = (quant && k < K) ? g.codes[k] : nullptr;
    p.s.p[k] = (quant && k < K) ? g.scales[k] : nullptr;
    p.o.p[k] = (hp.quant_offset && k < K) ? g.offsets[k] : nullptr;
    p.e.p[k] = (hp.error_feedback && k < K) ? g.residuals[k] : nullptr;
  }
}

static QuantForm form_of(const mlc_outer_group& g, const mlc_outer_hparams& hp) {
  return make_quant_form(hp.quant_bits, hp.quant_offset, hp.quant_per_matrix ? g.m : 0, hp.ef_beta);
}

int muloco_quantize_delta(const mlc_outer_group* groups, int n_groups, const mlc_outer_hparams* hp,
                          void* stream_) {
  int rc = check_outer(groups, n_groups, hp, false);
  if (rc != MLC_OK) return rc;
  if (hp->quant_bits == 0) return MLC_ERR_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  for (int i = 0; i < n_groups; ++i) {
    const mlc_outer_group& g = groups[i];
    OuterPtrs p;
    gather_ptrs(g, *hp, p);
    const QuantForm form = form_of(g, *hp);
    if (hp->quant_per_matrix) {
      rc = launch_matrix_ranges(p.w, g.worker_dtype, g.global_param, g.global_dtype, p.s, p.o, p.e, g.count,
                                g.m, g.n, hp->K, form, stream);
      if (rc != MLC_OK) return rc;
    }
    rc = launch_quantize(p.w, g.worker_dtype, g.global_param, g.global_dtype, p.c, p.s, p.o, p.e,
                         g.count * g.m, g.n, hp->K, form, stream);
    if (rc != MLC_OK) return rc;
  }
  return MLC_OK;
}

// Can this group go into a launch that covers several groups?
static bool multi_launch_covers(const mlc_outer_group& g, const mlc_outer_hparams& hp) {
  if (hp.K > OUTER_MAX_SEG_K || hp.second_quantisation || hp.quant_per_matrix) return false;
  if (hp.quant_bits == 0) return true;
  const int cfg = quant_reg_cfg(g.n);
  return cfg >= 0 && cfg <= QUANT_MULTI_MAX_CFG && !(g.worker_dtype == MLC_F32 && g.global_dtype == MLC_BF16);
}

int muloco_outer_step(const mlc_outer_group* groups, int n_groups, const mlc_outer_hparams* hp,
                      void* stream_) {
  int rc = check_outer(groups, n_groups, hp, true);
  if (rc != MLC_OK) return rc;
  hipStream_t stream = (hipStream_t)stream_;
  for (int i = 0; i < n_groups; ++i) {
    // Consecutive groups of one dtype pair share a launch (a streaming fragment of one layer
    // is three small groups: one launch instead of three fills the chip for longer).
    int run = 0;
    while (i + run < n_groups && run < OUTER_MAX_SEG && groups[i + run].worker_dtype == groups[i].worker_dtype &&
           groups[i + run].global_dtype == groups[i].global_dtype && multi_launch_covers(groups[i + run], *hp))
      ++run;
    if (run >= 2) {
      OuterGroupArgs args[OUTER_MAX_SEG];
      for (int j = 0; j < run; ++j) {
        const mlc_outer_group& g = groups[i + j];
        OuterPtrs p;
        gather_ptrs(g, *hp, p);
        args[j].w = p.w; args[j].codes = p.c; args[j].scales = p.s; args[j].offsets = p.o; args[j].ef = p.e;
        args[j].theta_g = g.global_param; args[j].u = g.outer_momentum;
        args[j].rows = g.count * g.m; args[j].n = g.n;
      }
      if (hp->quant_bits)
        rc = launch_quantize_outer_multi(args, run, groups[i].worker_dtype, groups[i].global_dtype, hp->K,
                                         form_of(groups[i], *hp), hp->eta_out, hp->mu, hp->nesterov,
                                         hp->write_back, stream);
      else
        rc = launch_outer_fused_multi(args, run, groups[i].worker_dtype, groups[i].global_dtype, hp->K,
                                      hp->eta_out, hp->mu, hp->nesterov, hp->write_back, stream);
      if (rc != MLC_OK) return rc;
      i += run - 1;
      continue;
    }
    const mlc_outer_group& g = groups[i];
    OuterPtrs p;
    gather_ptrs(g, *hp, p);
    if (hp->quant_bits) {
      const QuantForm form = form_of(g, *hp);
      if (hp->quant_per_matrix) {
        rc = launch_matrix_ranges(p.w, g.worker_dtype, g.global_param, g.global_dtype, p.s, p.o, p.e,
                                  g.count, g.m, g.n, hp->K, form, stream);
        if (rc != MLC_OK) return rc;
      }
      // one pass when the row fits in registers, else quantise and then consume the codes
      rc = launch_quantize_outer_fused(p.w, g.worker_dtype, g.global_param, g.global_dtype,
                                       g.outer_momentum, p.c, p.s, p.o, p.e, g.count * g.m, g.n, hp->K,
                                       form, hp->eta_out, hp->mu, hp->nesterov, hp->write_back,
                                       hp->second_quantisation,
                                       hp->second_quantisation ? g.mean_codes : nullptr,
                                       hp->second_quantisation ? g.mean_scales : nullptr,
                                       hp->second_quantisation ? g.mean_offsets : nullptr, stream);
      if (rc != MLC_ERR_UNSUPPORTED || hp->second_quantisation) {
        if (rc != MLC_OK) return rc;
        continue;
      }
      rc = launch_quantize(p.w, g.worker_dtype, g.global_param, g.global_dtype, p.c, p.s, p.o, p.e,
                           g.count * g.m, g.n, hp->K, form, stream);
      if (rc != MLC_OK) return rc;
      rc = launch_dequant_outer(p.w, g.worker_dtype, g.global_param, g.global_dtype, g.outer_momentum,
                                p.c, p.s, p.o, g.count * g.m, g.n, hp->K, form, hp->eta_out, hp->mu,
                                hp->nesterov, hp->write_back, stream);
    } else {
      rc = launch_outer_fused(p.w, g.worker_dtype, g.global_param, g.global_dtype, g.outer_momentum,
                              g.count * g.m * g.n, hp->K, hp->eta_out, hp->mu, hp->nesterov,
                              hp->write_back, stream);
    }
    if (rc != MLC_OK) return rc;
  }
  return MLC_OK;
}

size_t muloco_topk_workspace_bytes(const mlc_outer_group* groups, int n_groups, int K) {
  if (!groups || n_groups < 0 || K < 1 || K > MLC_MAX_WORKERS) return 0;
  size_t need = 0;
  for (int i = 0; i < n_groups; ++i) {
    if (groups[i].count < 1) return 0;
    const size_t b = topk_workspace_bytes(groups[i].count, K);
    if (b > need) need = b;
  }
  return need;
}

int muloco_topk_outer_step(const mlc_outer_group* groups, int n_groups, const mlc_outer_hparams* hp,
                           double fraction, void* workspace, size_t workspace_bytes, void* stream_) {
  int rc = check_outer(groups, n_groups, hp, true, true);
  if (rc != MLC_OK) return rc;
  if (!(fraction > 0.0) || fraction > 1.0) return MLC_ERR_ARG;
  if (hp->second_quantisation || hp->quant_offset || hp->quant_per_matrix) return MLC_ERR_ARG;
  if (n_groups == 0) return MLC_OK;
  if (!workspace || ((uintptr_t)workspace & 15)) return MLC_ERR_WORKSPACE;
  if (workspace_bytes < muloco_topk_workspace_bytes(groups, n_groups, hp->K)) return MLC_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  for (int i = 0; i < n_groups; ++i) {
    const mlc_outer_group& g = groups[i];
    if (g.count > 65535 || (double)g.m * (double)g.n >= 4294967296.0) return MLC_ERR_SHAPE;
    if (g.scales)
      for (int k = 0; k < hp->K; ++k)
        if (!g.scales[k] || !aligned16(g.scales[k])) return MLC_ERR_ARG;
  }
  for (int i = 0; i < n_groups; ++i) {
    const mlc_outer_group& g = groups[i];
    WorkerPtrs w; ScalePtrs t; ResidualPtrs e;
    for (int k = 0; k < MLC_MAX_WORKERS; ++k) {
      w.p[k] = k < hp->K ? g.worker_params[k] : nullptr;
      t.p[k] = (g.scales && k < hp->K) ? g.scales[k] : nullptr;
      e.p[k] = (hp->error_feedback && k < hp->K) ? g.residuals[k] : nullptr;
    }
    const double elems = (double)g.m * (double)g.n;
    double kc = std::ceil(fraction * elems);
    if (kc < 1.0) kc = 1.0;
    if (kc > elems) kc = elems;
    rc = launch_topk_outer(w, g.worker_dtype, g.global_param, g.global_dtype, g.outer_momentum, e, t,
                           g.count, g.m, g.n, hp->K, (unsigned int)kc, hp->ef_beta, hp->eta_out, hp->mu,
                           hp->nesterov, hp->write_back, workspace, stream);
    if (rc != MLC_OK) return rc;
  }
  return MLC_OK;
}

int muloco_adamw_step(const mlc_adamw_group* groups, int n_groups, const mlc_adamw_hparams* hp,
                      void* stream_) {
  if (!groups || !hp) return MLC_ERR_NULL;
  if (n_groups < 0) return MLC_ERR_ARG;
  if (!(hp->lr >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) ||
      !(hp->eps >= 0.f) || !(hp->weight_decay >= 0.f))
    return MLC_ERR_ARG;
  if (hp->bias_correction != 0 && hp->bias_correction != 1) return MLC_ERR_ARG;
  if (hp->bias_correction && hp->step < 1) return MLC_ERR_ARG;
  for (int i = 0; i < n_groups; ++i) {
    const mlc_adamw_group& g = groups[i];
    if (!g.param || !g.grad || !g.exp_avg || !g.exp_avg_sq) return MLC_ERR_NULL;
    if (!valid_dtype(g.param_dtype) || !valid_dtype(g.grad_dtype)) return MLC_ERR_DTYPE;
    if (g.count < 1 || g.count > ((int64_t)1 << 40)) return MLC_ERR_SHAPE;
    if (!aligned16(g.param) || !aligned16(g.grad) || !aligned16(g.exp_avg) || !aligned16(g.exp_avg_sq))
      return MLC_ERR_ARG;
  }
  float c1 = 1.f, c2 = 1.f;
  if (hp->bias_correction) {
    c1 = (float)(1.0 / (1.0 - std::pow((double)hp->beta1, (double)hp->step)));
    c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)hp->beta2, (double)hp->step)));
  }
  hipStream_t stream = (hipStream_t)stream_;
  for (int i = 0; i < n_groups; ++i) {
    const mlc_adamw_group& g = groups[i];
    const int rc = launch_adamw(g.param, g.param_dtype, g.grad, g.grad_dtype, g.exp_avg, g.exp_avg_sq,
                                g.count, hp->lr, hp->beta1, hp->beta2, hp->eps,
                                hp->lr * hp->weight_decay, c1, c2, stream);
    if (rc != MLC_OK) return rc;
  }
  return MLC_OK;
}

int muloco_timing_enable(int on) {
  TimingState& t = timing();
  std::lock_guard<std::mutex> lock(t.mu);
  t.enabled = on != 0;
  return MLC_OK;
}

int muloco_timing_read(mlc_kernel_timing* out) {
  if (!out) return MLC_ERR_NULL;
  TimingState& t = timing();
  std::lock_guard<std::mutex> lock(t.mu);
  for (int i = 0; i < MLC_KERNEL_FAMILIES; ++i) out[i] = mlc_kernel_timing{0, 0.0, 0.0, 0.0};
  int rc = MLC_OK;
  for (const TimingRecord& r : t.records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess ||
        hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
      rc = MLC_ERR_LAUNCH;
    } else if (r.family >= 0 && r.family < MLC_KERNEL_FAMILIES) {
      out[r.family].launches += 1;
      out[r.family].total_ms += ms;
      out[r.family].flops += r.flops;
      out[r.family].bytes += r.bytes;
    }
    t.pool.push_back(r.start);
    t.pool.push_back(r.stop);
  }
  t.records.clear();
  return rc;
}

}  // extern "C"
