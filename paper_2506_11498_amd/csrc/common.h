// Internal declarations shared by the LRSA kernels and the C-ABI dispatch (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lrsa {

// Problem description after validation: the ABI struct plus the derived partition
// (sink, P full chunks of the lag size, tail R, nq query chunks, Ns scored chunks).
struct Dims {
    int B, Hq, Hkv, G, n, d;
    int S, L, K, ddof, lp;
    int P, R, nq, Ns;
    float scale;
    int dtype;  // 0 fp32, 1 bf16
    int compact;  // MFMA attention kernels read a condensed copy of the gather list's K/V rows
    int64_t qs[3], ks[3];
    // Attention over a window of query rows (one "filling" step of m chunks): rows [row_begin, row_end), which
    // are the query chunks [fq0, fq1) plus the sink rows when row_begin == 0.  The whole sequence by default.
    int row_begin, row_end, fq0, fq1;
    int64_t lse_stride;   // floats between the lse (and D) rows of consecutive (batch, query head) pairs
    int acc;              // backward adds dK, dV into fp32 accumulators instead of writing them
};

// Number of entries of the gather list "sink ++ survivors of chunks 0..c-1" and the first
// position of the contiguous (fully kept) window, for a query in chunk q (q < 0: sink query).
__host__ __device__ inline int gather_count(const Dims& D, int q) {
    if (q < 0) return 0;
    int c = q - D.lp;
    return D.S + D.K * (c > 0 ? c : 0);
}
__host__ __device__ inline int window_start(const Dims& D, int q) {
    if (q < 0) return 0;
    int c = q - D.lp;
    return D.S + D.L * (c > 0 ? c : 0);
}

// ---- launchers (each enqueues on `st` and returns the first HIP error) ----------------------
size_t score_ws_bytes(const Dims&);
int score_route(const Dims&);
hipError_t launch_score(const Dims&, const void* K, const void* V, float* score, void* ws, hipStream_t st);

hipError_t launch_softmax_select(const Dims&, const float* sigma, float* score, int32_t* idx, hipStream_t st);
bool score_resident_applies(const Dims&);
int score_poll_limit(int polls);
hipError_t launch_score_resident(const Dims&, const void* K, const void* V, float* score, int32_t* idx, float* sigma,
                                 hipStream_t st);

size_t select_ws_bytes(const Dims&);
hipError_t launch_select(const Dims&, const float* score, int32_t* idx, void* ws, hipStream_t st);
hipError_t launch_check_idx(const Dims&, const int32_t* idx, int32_t* bad_rows, hipStream_t st);
size_t decode_ws_bytes(const Dims&);
bool cache_compress_supported(const Dims&);
hipError_t launch_cache_compress(const Dims&, void* Kc, void* Vc, int32_t* pos, int len, int done, int steps, hipStream_t st);
hipError_t launch_decode_attn(const Dims&, const void* q, const void* Kc, const void* Vc, int len, void* O, float* lse,
                              void* ws, hipStream_t st);
// lrsa_decode_attn_static: bytes of the library-owned scratch array and what a call needs of it
constexpr size_t DECODE_STATIC_SCRATCH_BYTES = size_t(4) << 20;
size_t decode_static_need(const Dims&, int len);
hipError_t launch_decode_attn_static(const Dims&, const void* q, const void* Kc, const void* Vc, int len, void* O,
                                     float* lse, hipStream_t st);
hipError_t launch_score_select(const Dims&, const void* K, const void* V, float* score, int32_t* idx, void* ws, hipStream_t st);

size_t attn_fwd_generic_ws_bytes(const Dims&);
hipError_t launch_attn_fwd_generic(const Dims&, const void* Q, const void* K, const void* V, const int32_t* idx,
                                   void* O, float* lse, void* ws, hipStream_t st);
size_t attn_bwd_generic_ws_bytes(const Dims&);
hipError_t launch_attn_bwd_generic(const Dims&, const void* Q, const void* K, const void* V, const void* O,
                                   const void* dO, const float* lse, const int32_t* idx, void* dQ, void* dK,
                                   void* dV, void* ws, hipStream_t st);

bool mfma_supported(const Dims&);
size_t attn_fwd_mfma_ws_bytes(const Dims&);
hipError_t launch_attn_fwd_mfma(const Dims&, const void* Q, const void* K, const void* V, const int32_t* idx,
                                void* O, float* lse, void* ws, hipStream_t st);
size_t attn_bwd_mfma_ws_bytes(const Dims&);
hipError_t launch_attn_bwd_mfma(const Dims&, const void* Q, const void* K, const void* V, const void* O,
                                const void* dO, const float* lse, const int32_t* idx, void* dQ, void* dK,
                                void* dV, float* accK, float* accV, void* ws, hipStream_t st);
hipError_t launch_bwd_acc_finish(const Dims&, const float* accK, const float* accV, void* dK, void* dV, hipStream_t st);

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Brackets one kernel launch with HIP events on its stream when timing is switched on
// (lrsa_timing_enable); does nothing otherwise.
class ScopedKernelTimer {
  public:
    ScopedKernelTimer(const char* name, hipStream_t st);
    ~ScopedKernelTimer();
  private:
    hipStream_t st_;
    int slot_;
};
#define LRSA_TIMED_LAUNCH(name, st, ...)            \
    do {                                            \
        ::lrsa::ScopedKernelTimer timer_(name, st); \
        hipLaunchKernelGGL(__VA_ARGS__);            \
    } while (0)

// ---- device helpers ---------------------------------------------------------------------------
#if defined(__HIPCC__)
typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(uint32_t(x) << 16); }
// round to nearest even (inputs are finite)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return bf16_t(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int VEC = 4;  // elements per 16-byte load
    __device__ static __forceinline__ void load(const float* p, float (&out)[4]) {
        float4 v = *reinterpret_cast<const float4*>(p);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
    __device__ static __forceinline__ float get(const float* p) { return *p; }
    __device__ static __forceinline__ void put(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ void load(const bf16_t* p, float (&out)[8]) {
        uint4 v = *reinterpret_cast<const uint4*>(p);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static __forceinline__ float get(const bf16_t* p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ void put(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
#endif

}  // namespace lrsa
