// C ABI of libdistr_attn.so: argument checks, workspace, launches. See include/distr_attn.h.
#include "../../include/distr_attn.h"

#include <cstdlib>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <vector>

#include "da_common.h"

namespace {

thread_local char g_err[256] = "";
std::atomic<void*> g_stream{nullptr};

constexpr int kMaxDevices = 16;
std::mutex g_ws_mutex;
void* g_ws_ptr[kMaxDevices] = {nullptr};     // library-owned workspace, one per device
size_t g_ws_bytes[kMaxDevices] = {0};
// Buffers the library-owned workspace has outgrown. Work enqueued by earlier calls (or by a
// thread that fetched the pointer just before the growth) may still use them, so they are kept
// until distr_attn_release instead of being freed inside a forward call.
std::vector<void*> g_ws_retired[kMaxDevices];

// Scratch of distr_attn_fwd_noalloc: a fixed device array, one copy per GPU the library is
// loaded on, resident until the process ends. Host code never uses the array's name as an
// address: the per-device address comes from hipGetSymbolAddress (static_scratch below).
constexpr size_t kStaticScratchBytes = (size_t)DISTR_ATTN_NOALLOC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

struct Resolved {
  da::Problem pb;
  int dtype;
  int Tq;        // query blocks per head
  int Tk_side;   // K blocks per head whose groupings the mirrored form (side 1) uses
  hipStream_t stream;
};

// Checks shared by every entry point. need_groups: the call uses the LSH grouping.
int resolve(const da_params* p, bool need_groups, Resolved* out) {
  if (!p) return fail(DA_ERR_INVALID_ARG, "params is null");
  if (p->B <= 0 || p->H <= 0 || p->Hkv <= 0 || p->N <= 0 || p->d <= 0 || p->Br <= 0 || p->Bc <= 0)
    return fail(DA_ERR_INVALID_ARG, "B, H, Hkv, N, d, Br, Bc must be positive");
  if (p->H % p->Hkv != 0) return fail(DA_ERR_INVALID_ARG, "H (%d) is not a multiple of Hkv (%d)", p->H, p->Hkv);
  if (p->dtype != DA_BF16 && p->dtype != DA_F32) return fail(DA_ERR_INVALID_ARG, "unknown dtype %d", p->dtype);
  if (p->causal != 0 && p->causal != 1) return fail(DA_ERR_INVALID_ARG, "causal must be 0 or 1");
  if (p->Nk < 0) return fail(DA_ERR_INVALID_ARG, "Nk must be positive, or 0 for Nk = N");
  const int Nk = p->Nk > 0 ? p->Nk : p->N;
  if (p->causal && Nk < p->N)
    return fail(DA_ERR_INVALID_ARG, "causal with Nk (%d) < N (%d): the first queries would see no key", Nk, p->N);
  if (p->side != 0 && p->side != 1) return fail(DA_ERR_INVALID_ARG, "side must be 0 or 1");
  int n_planes = p->n_planes == 0 ? 16 : p->n_planes;
  if (need_groups) {
    if (p->n_groups <= 0 || p->d % p->n_groups != 0)
      return fail(DA_ERR_INVALID_ARG, "n_groups (%d) must divide d (%d): groups have a constant size", p->n_groups, p->d);
    if (n_planes < 1) return fail(DA_ERR_INVALID_ARG, "n_planes must be positive");
    if (p->gray_mode != 0 && p->gray_mode != 1) return fail(DA_ERR_INVALID_ARG, "gray_mode must be 0 or 1");
  }
  float scale = p->softmax_scale;
  if (scale == 0.0f) scale = 1.0f / std::sqrt((float)p->d);
  if (!(scale > 0.0f) || !std::isfinite(scale)) return fail(DA_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
  if ((long long)p->B * p->H * ((p->N + p->Br - 1) / p->Br) > 0x7fffffffLL)
    return fail(DA_ERR_UNSUPPORTED, "more than 2^31-1 query blocks");
  // limits of the kernels
  const long long n_max = p->N > Nk ? p->N : Nk;
  if (n_max * p->d * 4 > 0x7fffffffLL)
    return fail(DA_ERR_UNSUPPORTED, "N * d = %lld: one head must stay below 2 GiB (32-bit tile offsets)", n_max * p->d);
  if (p->d != 64 && p->d != 128) return fail(DA_ERR_UNSUPPORTED, "d = %d: kernels are built for d in {64, 128}", p->d);
  if (p->Br != 64 && p->Br != 128 && p->Br != 256)
    return fail(DA_ERR_UNSUPPORTED, "Br = %d: kernels are built for Br in {64, 128, 256}", p->Br);
  const bool mirrored = need_groups && p->side == 1;
  if (mirrored) {
    if (p->Bc != 32 && p->Bc != 64 && p->Bc != 128)
      return fail(DA_ERR_UNSUPPORTED, "Bc = %d: side = 1 groups K blocks of 32, 64 or 128 rows", p->Bc);
  } else if (p->Bc != 32 && p->Bc != 64 && p->Bc != 128) {
    return fail(DA_ERR_UNSUPPORTED, "Bc = %d: kernels are built for Bc in {32, 64, 128}", p->Bc);
  }
  if (p->lse_out) {
    if (mirrored) return fail(DA_ERR_UNSUPPORTED, "lse_out is not written by the mirrored form (side = 1)");
    if (((uintptr_t)p->lse_out & 3u) != 0) return fail(DA_ERR_INVALID_ARG, "lse_out must be 4-byte aligned");
  }
  if (need_groups && n_planes > da::kMaxPlanes) return fail(DA_ERR_UNSUPPORTED, "n_planes = %d > %d", n_planes, da::kMaxPlanes);
  out->pb = da::Problem{p->B, p->H, p->Hkv, p->N, p->d, p->Br, need_groups ? p->n_groups : p->d,
                        p->causal, n_planes, p->gray_mode, p->lsh_seed, scale, Nk, mirrored ? 1 : 0, p->Bc, p->lse_out};
  out->dtype = p->dtype;
  out->Tq = (p->N + p->Br - 1) / p->Br;
  out->Tk_side = (Nk + p->Bc - 1) / p->Bc;
  out->stream = (hipStream_t)(p->stream ? p->stream : g_stream.load());
  return DA_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int check_tensors(const void* q, const void* k, const void* v, const void* o) {
  if (!q || !k || !v || !o) return fail(DA_ERR_INVALID_ARG, "q, k, v, o must be non-null");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
    return fail(DA_ERR_INVALID_ARG, "q, k, v, o must be 16-byte aligned");
  if (o == q || o == k || o == v) return fail(DA_ERR_INVALID_ARG, "o must not alias an input");
  return DA_OK;
}

// Table of groupings: one row of d channels per Q block, or per K block for the mirrored form.
size_t perm_bytes(const Resolved& r) {
  size_t n = r.pb.side == 1 ? (size_t)r.pb.B * r.pb.Hkv * r.Tk_side * r.pb.d
                            : (size_t)r.pb.B * r.pb.H * r.Tq * r.pb.d;
  return (n + 255) & ~(size_t)255;
}

// The LSH stage as the mirrored form needs it: over K, one block of Bc rows at a time.
da::Problem key_side_problem(const da::Problem& pb) {
  da::Problem k = pb;
  k.H = pb.Hkv;
  k.N = pb.Nk;
  k.Br = pb.Bc;
  return k;
}

// Transposed half-precision copy of K that the bf16 distr path reads: [B][Hkv][d][Npad].
size_t kt_bytes(const Resolved& r) {
  if (r.dtype != DA_BF16) return 0;
  return da::kt_copy_bytes(r.pb.B, r.pb.Hkv, r.pb.d, r.pb.Nk) + da::kRtabBytes;
}

// The transposed copy of K is read by the bf16 matrix-core kernels (the mirrored form runs on the
// float-arithmetic kernel and needs none).
bool needs_kt(const Resolved& r) { return r.dtype == DA_BF16 && r.pb.side == 0; }

// Address of the static scratch array on the current device (looked up once per device).
int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fail(DA_ERR_HIP, "hipGetDevice failed");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(DA_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DA_OK;
}

// Device scratch of the distr path: [K^T copy | permutation table]. Only the parts this call
// writes are asked for: no K^T copy when the caller brings kt_in (or on the float path), no
// table when the grouping comes from perm_in, goes to perm_out, or stays inside the attention
// kernel. Source: the caller's workspace, the static array (no_alloc), or the library-owned buffer.
int scratch_base(const da_params* p, const Resolved& r, size_t need, bool no_alloc, char** out) {
  char* base = nullptr;
  if (no_alloc) {
    if (need > kStaticScratchBytes)
      return fail(DA_ERR_WORKSPACE, "distr_attn_fwd_noalloc: %zu bytes of scratch needed, the static array holds %zu "
                  "(pass kt_in, or use distr_attn_fwd_ex with a workspace)", need, kStaticScratchBytes);
    void* ptr = nullptr;
    int rc = static_scratch(&ptr);
    if (rc) return rc;
    base = (char*)ptr;
  } else if (p->workspace) {
    if (p->workspace_bytes < need)
      return fail(DA_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", p->workspace_bytes, need);
    if (((uintptr_t)p->workspace & 255u) != 0) return fail(DA_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    base = (char*)p->workspace;
  } else {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fail(DA_ERR_HIP, "hipGetDevice failed");
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (g_ws_bytes[dev] < need) {
      // Growing allocates: not allowed while the stream is being captured into a graph.
      hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
      if (hipStreamIsCapturing(r.stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
        return fail(DA_ERR_WORKSPACE, "the library-owned workspace would have to grow to %zu bytes while the stream is "
                    "being captured: pass a workspace, or run the call once before capturing", need);
      void* ptr = nullptr;
      hipError_t e = hipMalloc(&ptr, need);
      if (e != hipSuccess) return fail(DA_ERR_WORKSPACE, "hipMalloc(%zu) failed: %s", need, hipGetErrorString(e));
      if (g_ws_ptr[dev]) g_ws_retired[dev].push_back(g_ws_ptr[dev]);
      g_ws_ptr[dev] = ptr;
      g_ws_bytes[dev] = need;
    }
    base = (char*)g_ws_ptr[dev];
  }
  *out = base;
  return DA_OK;
}

int get_scratch(const da_params* p, const Resolved& r, bool need_table, bool no_alloc, uint8_t** perm, void** kt) {
  const size_t kt_need = (needs_kt(r) && !p->kt_in) ? kt_bytes(r) : 0;
  const size_t perm_need = need_table ? perm_bytes(r) : 0;
  const size_t need = kt_need + perm_need;
  char* base = nullptr;
  if (need == 0) {
    *kt = nullptr;
    *perm = nullptr;
    return DA_OK;
  }
  int rc = scratch_base(p, r, need, no_alloc, &base);
  if (rc) return rc;
  *kt = kt_need ? (void*)base : nullptr;
  *perm = perm_need ? (uint8_t*)(base + kt_need) : nullptr;
  return DA_OK;
}

// Scratch of the backward pass: [permutation table, when the LSH stage runs and the table is not
// exported | what the bf16 kernels keep between their launches (D_i, Q~)].
size_t bwd_tail_bytes(const Resolved& r, bool distr) {
  return r.dtype == DA_BF16 ? da::attn_bf16_bwd_scratch_bytes(r.pb, distr ? 1 : 0) : 0;
}

// DISTR_ATTN_DEBUG=1 in the environment (read once): wait for the device after every launch, so
// that a fault is reported by the call and the launch that caused it.
bool debug_sync() {
  static const bool on = [] {
    const char* v = std::getenv("DISTR_ATTN_DEBUG");
    return v != nullptr && v[0] == '1';
  }();
  return on;
}

int check_launch(hipError_t e, const char* what, hipStream_t stream) {
  if (e != hipSuccess) return fail(DA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (debug_sync() && hipStreamIsCapturing(stream, &cap) == hipSuccess && cap == hipStreamCaptureStatusNone) {
    const hipError_t s = hipDeviceSynchronize();
    if (s != hipSuccess) return fail(DA_ERR_HIP, "%s (found by DISTR_ATTN_DEBUG): %s", what, hipGetErrorString(s));
  }
  return DA_OK;
}

int attention(const void* q, const void* k, const void* v, void* o, const da_params* p, bool distr,
              bool no_alloc = false) {
  Resolved r;
  int rc = resolve(p, distr, &r);
  if (rc) return rc;
  rc = check_tensors(q, k, v, o);
  if (rc) return rc;
  if (r.dtype == DA_BF16 && r.pb.side == 0 && !da::attn_bf16_supported(r.pb, distr ? 1 : 0))
    return fail(DA_ERR_UNSUPPORTED, "bf16 kernels need n_groups in {4, 8, 16, 32, 64, 128} (16, 32, 64 or d when Bc is not "
                "64) and groups of at most 16 channels; got d=%d Br=%d Bc=%d n_groups=%d", p->d, p->Br, p->Bc, p->n_groups);
  const uint8_t* perm = nullptr;
  void* kt = nullptr;
  // Groups of one channel (G* = 1): S^ = Q_r K_f^T is Q K^T with its terms taken in the sorted
  // channel order (Sec. 3.1: one column per group reproduces S). The bf16 path then runs the
  // exact kernel; the LSH stage still runs if the caller asked for its tables.
  const bool trivial_groups = distr && r.dtype == DA_BF16 && r.pb.side == 0 && p->n_groups == p->d;
  if (trivial_groups) {
    if (!p->perm_in && (p->perm_out || p->hash_out)) {
      rc = check_launch(da::launch_lsh_group(q, r.dtype, r.pb, p->perm_out, p->hash_out, r.stream), "lsh_group launch", r.stream);
      if (rc) return rc;
    }
    distr = false;
  }
  if (distr) {
    // bf16 path, up to 16 projections, no hashes asked for: the attention kernel hashes and groups
    // its own Q block in its prologue (same arithmetic as the LSH kernel); the table is written
    // only if the caller gave perm_out.
    const bool lsh_in_kernel = r.dtype == DA_BF16 && r.pb.side == 0 && !p->perm_in && !p->hash_out && r.pb.n_planes <= 16;
    if (lsh_in_kernel) r.pb.perm_w = p->perm_out;
    const bool run_lsh = !p->perm_in && !lsh_in_kernel;
    uint8_t* table = nullptr;
    rc = get_scratch(p, r, run_lsh && !p->perm_out, no_alloc, &table, &kt);
    if (rc) return rc;
    if (p->perm_in) {
      perm = p->perm_in;
    } else if (run_lsh) {
      if (p->perm_out) table = p->perm_out;
      rc = check_launch(r.pb.side == 1
                            ? da::launch_lsh_group(k, r.dtype, key_side_problem(r.pb), table, p->hash_out, r.stream)
                            : da::launch_lsh_group(q, r.dtype, r.pb, table, p->hash_out, r.stream),
                        "lsh_group launch", r.stream);
      if (rc) return rc;
      perm = table;
    }
    if (needs_kt(r) && p->kt_in) {
      if (((uintptr_t)p->kt_in & 255u) != 0) return fail(DA_ERR_INVALID_ARG, "kt_in must be 256-byte aligned");
      kt = const_cast<void*>(p->kt_in);
    } else if (needs_kt(r)) {
      rc = check_launch(da::launch_kt_prepass(k, kt, r.pb, r.stream), "key pre-pass launch", r.stream);
      if (rc) return rc;
    }
  }
  // (the mirrored form runs on the float-arithmetic kernel for either dtype)
  hipError_t e = (r.dtype == DA_BF16 && !(distr && r.pb.side == 1))
                     ? da::launch_attn_bf16(q, k, v, o, perm, kt, r.pb, distr ? 1 : 0, r.stream)
                     : da::launch_attn_f32(q, k, v, o, perm, r.pb, r.dtype, distr ? 1 : 0, r.stream);
  return check_launch(e, "attention launch", r.stream);
}

// Backward of the float path. The grouping is the forward's: the LSH stage runs again on q with
// the same parameters (or the caller's perm_in is used), then the two gradient kernels.
int attention_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                  void* dq, void* dk, void* dv, const da_params* p, bool distr) {
  Resolved r;
  int rc = resolve(p, distr, &r);
  if (rc) return rc;
  if (r.pb.side == 1) return fail(DA_ERR_UNSUPPORTED, "the backward pass is built for side = 0 only");
  if (r.dtype == DA_BF16 && ((size_t)r.pb.N * r.pb.d * 2 >= 0x7fffffffULL || (size_t)r.pb.Nk * r.pb.d * 2 >= 0x7fffffffULL))
    return fail(DA_ERR_UNSUPPORTED, "a head of 2 GiB or more: the backward kernels address tiles by 32-bit byte offsets");
  const void* in[] = {q, k, v, o, dout, lse};
  void* out[] = {dq, dk, dv};
  for (const void* x : in)
    if (!x || !aligned16(x)) return fail(DA_ERR_INVALID_ARG, "q, k, v, o, dout, lse must be non-null and 16-byte aligned");
  for (void* y : out) {
    if (!y || !aligned16(y)) return fail(DA_ERR_INVALID_ARG, "dq, dk, dv must be non-null and 16-byte aligned");
    for (const void* x : in)
      if (x == y) return fail(DA_ERR_INVALID_ARG, "dq, dk, dv must not alias an input");
  }
  if (dq == dk || dq == dv || dk == dv) return fail(DA_ERR_INVALID_ARG, "dq, dk, dv must be distinct buffers");
  const bool own_table = distr && !p->perm_in && !p->perm_out;
  const size_t table_need = own_table ? perm_bytes(r) : 0;
  const size_t tail_need = bwd_tail_bytes(r, distr);
  char* base = nullptr;
  if (table_need + tail_need) {
    rc = scratch_base(p, r, table_need + tail_need, false, &base);
    if (rc) return rc;
  }
  const uint8_t* perm = nullptr;
  if (distr) {
    if (p->perm_in) {
      perm = p->perm_in;
    } else {
      uint8_t* table = p->perm_out ? p->perm_out : (uint8_t*)base;
      rc = check_launch(da::launch_lsh_group(q, r.dtype, r.pb, table, p->hash_out, r.stream), "lsh_group launch", r.stream);
      if (rc) return rc;
      perm = table;
    }
  }
  if (r.dtype == DA_BF16)
    return check_launch(da::launch_attn_bf16_bwd(q, k, v, o, dout, lse, dq, dk, dv, perm, base + table_need, r.pb,
                                                 distr ? 1 : 0, r.stream),
                        "backward launch (matrix cores)", r.stream);
  return check_launch(da::launch_attn_f32_bwd(q, k, v, o, dout, lse, dq, dk, dv, perm, r.pb, distr ? 1 : 0, r.stream),
                      "backward launch", r.stream);
}

da_params short_form(int B, int H, int Hkv, int N, int d, int Br, int Bc, int n_groups, uint64_t seed, int causal) {
  da_params p = {};
  p.B = B; p.H = H; p.Hkv = Hkv; p.N = N; p.d = d; p.Br = Br; p.Bc = Bc;
  p.n_groups = n_groups; p.causal = causal; p.lsh_seed = seed;
  p.dtype = DA_BF16;
  return p;
}

}  // namespace

extern "C" {

int distr_attn_fwd(const void* q, const void* k, const void* v, void* o, int B, int H, int Hkv, int N,
                   int d, int Br, int Bc, int n_groups, uint64_t lsh_seed, int causal) {
  da_params p = short_form(B, H, Hkv, N, d, Br, Bc, n_groups, lsh_seed, causal);
  return attention(q, k, v, o, &p, true);
}

int distr_attn_exact_fwd(const void* q, const void* k, const void* v, void* o, int B, int H, int Hkv,
                         int N, int d, int Br, int Bc, int causal) {
  da_params p = short_form(B, H, Hkv, N, d, Br, Bc, d, 0, causal);
  return attention(q, k, v, o, &p, false);
}

int distr_attn_fwd_ex(const void* q, const void* k, const void* v, void* o, const da_params* p) {
  return attention(q, k, v, o, p, true);
}

int distr_attn_exact_fwd_ex(const void* q, const void* k, const void* v, void* o, const da_params* p) {
  return attention(q, k, v, o, p, false);
}

int distr_attn_bwd_ex(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                      void* dq, void* dk, void* dv, const da_params* p) {
  return attention_bwd(q, k, v, o, dout, lse, dq, dk, dv, p, true);
}

int distr_attn_exact_bwd_ex(const void* q, const void* k, const void* v, const void* o, const void* dout,
                            const float* lse, void* dq, void* dk, void* dv, const da_params* p) {
  return attention_bwd(q, k, v, o, dout, lse, dq, dk, dv, p, false);
}

int distr_attn_fwd_noalloc(const void* q, const void* k, const void* v, void* o, const da_params* p) {
  return attention(q, k, v, o, p, true, true);
}

size_t distr_attn_noalloc_max_bytes(void) { return kStaticScratchBytes; }

int distr_attn_lsh_group(const void* q, const da_params* p) {
  Resolved r;
  int rc = resolve(p, true, &r);
  if (rc) return rc;
  if (!q) return fail(DA_ERR_INVALID_ARG, "q must be non-null");
  if (!p->perm_out && !p->hash_out) return fail(DA_ERR_INVALID_ARG, "perm_out or hash_out must be given");
  // side 1: the tensor is K ([B][Hkv][Nk][d]) and the blocks are its Bc-row K blocks
  return check_launch(da::launch_lsh_group(q, r.dtype, r.pb.side == 1 ? key_side_problem(r.pb) : r.pb, p->perm_out,
                                           p->hash_out, r.stream), "lsh_group launch", r.stream);
}

int distr_attn_key_prepass(const void* k, void* kt_out, const da_params* p) {
  Resolved r;
  int rc = resolve(p, true, &r);
  if (rc) return rc;
  if (!k || !kt_out) return fail(DA_ERR_INVALID_ARG, "k and kt_out must be non-null");
  if (r.dtype != DA_BF16) return fail(DA_ERR_UNSUPPORTED, "the key pre-pass belongs to the bf16 path");
  if (((uintptr_t)k & 15u) != 0 || ((uintptr_t)kt_out & 255u) != 0)
    return fail(DA_ERR_INVALID_ARG, "k must be 16-byte and kt_out 256-byte aligned");
  return check_launch(da::launch_kt_prepass(k, kt_out, r.pb, r.stream), "key pre-pass launch", r.stream);
}

size_t distr_attn_kt_bytes(const da_params* p) {
  Resolved r;
  if (resolve(p, true, &r)) return 0;
  return kt_bytes(r);
}

size_t distr_attn_workspace_bytes(const da_params* p) {
  Resolved r;
  if (resolve(p, true, &r)) return 0;
  return (needs_kt(r) ? kt_bytes(r) : 0) + perm_bytes(r);
}

size_t distr_attn_bwd_workspace_bytes(const da_params* p) {
  Resolved r;
  if (resolve(p, true, &r)) return 0;
  return perm_bytes(r) + bwd_tail_bytes(r, true);
}

int distr_attn_hyperplanes(uint64_t seed, int n_planes, int Br, float* host_out) {
  if (!host_out || n_planes < 1 || n_planes > da::kMaxPlanes || Br < 1)
    return fail(DA_ERR_INVALID_ARG, "hyperplanes: bad arguments");
  for (int p = 0; p < n_planes; ++p)
    for (int r = 0; r < Br; ++r)
      host_out[(size_t)p * Br + r] = da::hyperplane_entry(seed, (uint32_t)p, (uint32_t)r);
  return DA_OK;
}

int distr_attn_set_stream(void* hip_stream) {
  g_stream.store(hip_stream);
  return DA_OK;
}

int distr_attn_release(void) {
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  int rc = DA_OK;
  int cur = 0;
  bool have_cur = hipGetDevice(&cur) == hipSuccess;
  for (int dev = 0; dev < kMaxDevices; ++dev) {
    if (!g_ws_ptr[dev] && g_ws_retired[dev].empty()) continue;
    bool ok = hipSetDevice(dev) == hipSuccess && hipDeviceSynchronize() == hipSuccess;
    if (ok && g_ws_ptr[dev]) ok = hipFree(g_ws_ptr[dev]) == hipSuccess;
    for (void* old : g_ws_retired[dev]) ok = ok && hipFree(old) == hipSuccess;
    if (!ok) rc = fail(DA_ERR_HIP, "release: freeing the workspace of device %d failed", dev);
    g_ws_retired[dev].clear();
    g_ws_ptr[dev] = nullptr;
    g_ws_bytes[dev] = 0;
  }
  if (have_cur) (void)hipSetDevice(cur);
  return rc;
}

const char* distr_attn_last_error(void) { return g_err; }

const char* distr_attn_version(void) { return "distr_attn 0.1 (gfx950)"; }

}  // extern "C"
