// Decode attention over the dense KV cache this library writes (paper Section 3.1, decode-attention
// paragraph: the present token's q/k/v are reconstructed once, the history is read from a standard
// dense cache [batch, position, head, head_dim]; Section 4: RoPE on q and k).
//
//   k_attn_decode    one workgroup per (token row, head, share of the visible positions): streams its
//                    share of K and V once (the step is bound by those bytes), online softmax per group
//                    of E/8 lanes, groups combined through LDS.  With one new token per sequence it also
//                    rotates its query and -- the workgroup whose share ends there -- the new key row.
//   k_attn_combine   folds the shares of one (row, head).  (A combine by the last workgroup to arrive,
//                    through device-coherent accesses and a counter, was measured slower than this
//                    second launch: the arrivals at one counter serialise.)
//   k_attn_prepare   only with several new tokens per sequence: rotates all new key rows in place first
//                    and writes the rotated queries to the workspace.
// A generic kernel (any head_dim, fp32 caches, fp64 arithmetic for fp32 data) covers what the fast one
// does not.
#include <stdlib.h>
#include "attention.hpp"

namespace lr {

size_t attn_ws_bytes(int64_t M, int64_t d, int64_t H) {
    const int64_t E = H > 0 ? d / H : 0;
    return kHeaderBytes + align256((size_t)M * (size_t)d * 8) +
           align256((size_t)M * (size_t)H * kAttnMaxSplit * (size_t)(E + 2) * 4);
}

AttnLayout attn_layout(void* ws, int64_t M, int64_t d, int64_t /*H*/) {
    AttnLayout L;
    char* p = (char*)ws + kHeaderBytes;
    L.q_rot = p; p += align256((size_t)M * (size_t)d * 8);
    L.part = (float*)p;
    return L;
}

bool attn_fast_ok(int dtype, int64_t E, bool aligned) {
    return dtype == LR_BF16 && aligned && (E == 64 || E == 128 || E == 256);
}

// element access by storage type
template <typename T> struct AIo;
template <> struct AIo<float> {
    __device__ static __forceinline__ float ld(const float* p) { return *p; }
    __device__ static __forceinline__ float cvt(double v) { return (float)v; }
};
template <> struct AIo<bf16_t> {
    __device__ static __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ bf16_t cvt(double v) { return f32_to_bf16((float)v); }
};

struct AttnArgs {
    const void* q; void* q_rot; void* k_cache; const void* v_cache; const int32_t* pos; void* out;
    float* part;
    int M, T, H, E, S_max, NS;
    float qscale;           // what the stored queries are multiplied by (fast path: scale * log2 e; generic: 1)
    float scale;
    double rope_base;       // <= 0: no rotation
};

// cos and sin of position * base^(-2i/E).  The angle is formed and reduced to [-pi, pi] in fp64 (a position of
// 10^5 times a relative error of 10^-7 would already be 10^-2 rad); for bf16 data the functions themselves are
// then evaluated in fp32, for fp32 data in fp64.
template <typename QR>
__device__ __forceinline__ void rope_cos_sin(long long p, int i, int E, double base, double& c, double& sn) {
    const double theta = exp2(-2.0 * (double)i / (double)E * log2(base));
    const double ang = (double)p * theta;
    if constexpr (sizeof(QR) == 8) {
        c = cos(ang); sn = sin(ang);
    } else {
        const double k = rint(ang * 0.15915494309189535);                    // 1 / (2 pi)
        const double red = fma(-k, 1.2246467991473532e-16 * 2.0, fma(-k, 6.283185307179586, ang));
        float sf, cf;
        sincosf((float)red, &sf, &cf);
        c = (double)cf; sn = (double)sf;
    }
}

// ---- prepare: rotate-half RoPE, pair (i, i + E/2), angle = position * base^(-2i/E), in fp64 ------
template <typename T, typename QR>
__global__ void __launch_bounds__(256) k_attn_prepare(AttnArgs a) {
    const int half = a.E >> 1;
    const long long total = (long long)a.M * a.H * half;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
        const int i = (int)(idx % half);
        const int h = (int)((idx / half) % a.H);
        const int r = (int)(idx / ((long long)half * a.H));
        const int b = r / a.T, s = r - b * a.T;
        const long long p = (long long)a.pos[b] + s;
        const size_t qo = (size_t)r * a.H * a.E + (size_t)h * a.E + i;
        const T* q = reinterpret_cast<const T*>(a.q);
        QR* qr = reinterpret_cast<QR*>(a.q_rot);
        double qlo = (double)AIo<T>::ld(q + qo), qhi = (double)AIo<T>::ld(q + qo + half);
        if (a.rope_base > 0.0) {
            double c, sn;
            rope_cos_sin<QR>(p, i, a.E, a.rope_base, c, sn);
            const double lo = qlo * c - qhi * sn, hi = qhi * c + qlo * sn;
            qlo = lo; qhi = hi;
            if (p >= 0 && p < a.S_max) {
                T* k = reinterpret_cast<T*>(a.k_cache) + (((size_t)b * a.S_max + (size_t)p) * a.H + h) * a.E + i;
                const double klo = (double)AIo<T>::ld(k), khi = (double)AIo<T>::ld(k + half);
                k[0] = AIo<T>::cvt(klo * c - khi * sn);
                k[half] = AIo<T>::cvt(khi * c + klo * sn);
            }
        }
        qr[qo] = (QR)(qlo * (double)a.qscale);
        qr[qo + half] = (QR)(qhi * (double)a.qscale);
    }
}

// ---- fast kernel ----------------------------------------------------------------------------------
__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// How the visible positions [0, n) of one (row, head) are shared: `ns` workgroups (at most NS, each with at
// least one sweep of KG positions), `per` positions each.  The same arithmetic runs in the main kernel and in
// the combine kernel.
__device__ __forceinline__ void split_of(int n, int NS, int KG, int& ns, int& per) {
    int want = (n + KG - 1) / KG;
    want = want < 1 ? 1 : (want > NS ? NS : want);
    per = (n + want - 1) / want;
    per = (per + KG - 1) / KG * KG;
    if (per < KG) per = KG;
    ns = (n + per - 1) / per;           // every share [sp * per, ...) with sp < ns starts below n
    if (ns < 1) ns = 1;
}

__device__ __forceinline__ int visible_positions(const AttnArgs& a, int b, int s) {
    const long long nn = (long long)a.pos[b] + s + 1;                 // causal
    return (int)(nn < 0 ? 0 : (nn > a.S_max ? a.S_max : nn));
}

// FUSED (one new token per sequence): the workgroup rotates its head's query itself, and the workgroup whose
// share ends at the new position rotates that key row in the cache; no prepare launch.  Otherwise the rotated,
// pre-scaled queries come from the workspace and the cache is already rotated.
template <int E, bool FUSED>
__global__ void __launch_bounds__(256) k_attn_decode(AttnArgs a) {
    constexpr int G = E / 8;            // lanes that share one cached position (16 bytes each)
    constexpr int KG = 256 / G;         // positions a workgroup takes per sweep = number of lane groups
    constexpr int UNR = 4;              // positions per group and sweep; two sweeps are in flight
    __shared__ float s_m[KG], s_l[KG];
    __shared__ float s_acc[KG][E];
    __shared__ float s_q[E], s_knew[E];
    const int tid = threadIdx.x, grp = tid / G, gl = tid % G;
    const int sp = blockIdx.x % a.NS, rh = blockIdx.x / a.NS;
    const int h = rh % a.H, r = rh / a.H;
    const int b = r / a.T, s = r - b * a.T;
    const int n = visible_positions(a, b, s);
    int ns, per;
    split_of(n, a.NS, KG, ns, per);
    if (sp >= ns) return;               // nothing for this workgroup (whole workgroup leaves)
    const int j0 = sp * per, j1 = (j0 + per < n) ? j0 + per : n;

    const size_t row_stride = (size_t)a.H * E;
    bf16_t* kbase = reinterpret_cast<bf16_t*>(a.k_cache) + ((size_t)b * a.S_max * a.H + h) * E;
    const bf16_t* kb = kbase + gl * 8;
    const bf16_t* vb = reinterpret_cast<const bf16_t*>(a.v_cache) + ((size_t)b * a.S_max * a.H + h) * E + gl * 8;
    const bool rope = a.rope_base > 0.0;
    const bool holds_new = FUSED && rope && j1 == n && n > 0;       // this share ends with the new token's key

    // first sweep's loads go out before anything else
    uint4 kk[UNR], vv[UNR];
    int j = j0 + grp;
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const int jj = j + u * KG;
        const int jc = jj < j1 ? jj : (j < j1 ? j : j0);             // positions past the end repeat a valid one; unused
        kk[u] = *reinterpret_cast<const uint4*>(kb + (size_t)jc * row_stride);
        vv[u] = *reinterpret_cast<const uint4*>(vb + (size_t)jc * row_stride);
    }

    float qv[8];
    if constexpr (FUSED) {
        if (tid < E / 2) {
            const bf16_t* q = reinterpret_cast<const bf16_t*>(a.q) + (size_t)r * a.H * E + (size_t)h * E;
            double qlo = (double)bf16_to_f32(q[tid]), qhi = (double)bf16_to_f32(q[tid + E / 2]);
            if (rope) {
                double c, sn;
                rope_cos_sin<float>((long long)n - 1, tid, E, a.rope_base, c, sn);
                const double lo = qlo * c - qhi * sn, hi = qhi * c + qlo * sn;
                qlo = lo; qhi = hi;
                if (holds_new) {
                    bf16_t* kn = kbase + (size_t)(n - 1) * row_stride;
                    const double klo = (double)bf16_to_f32(kn[tid]), khi = (double)bf16_to_f32(kn[tid + E / 2]);
                    const bf16_t rlo = f32_to_bf16((float)(klo * c - khi * sn)), rhi = f32_to_bf16((float)(khi * c + klo * sn));
                    kn[tid] = rlo; kn[tid + E / 2] = rhi;             // the cache keeps the rotated key
                    s_knew[tid] = bf16_to_f32(rlo); s_knew[tid + E / 2] = bf16_to_f32(rhi);
                }
            }
            s_q[tid] = (float)(qlo * (double)a.qscale); s_q[tid + E / 2] = (float)(qhi * (double)a.qscale);
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[e] = s_q[gl * 8 + e];
    } else {
        const float* q = reinterpret_cast<const float*>(a.q_rot) + (size_t)r * a.H * E + (size_t)h * E + gl * 8;
        const float4 q0 = *reinterpret_cast<const float4*>(q), q1 = *reinterpret_cast<const float4*>(q + 4);
        qv[0] = q0.x; qv[1] = q0.y; qv[2] = q0.z; qv[3] = q0.w; qv[4] = q1.x; qv[5] = q1.y; qv[6] = q1.z; qv[7] = q1.w;
    }

    float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (; j < j1; j += KG * UNR) {
        // next sweep's loads fly while this one is used
        uint4 kn[UNR], vn[UNR];
        const int jn = j + KG * UNR;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int jj = jn + u * KG;
            const int jc = jj < j1 ? jj : j;
            kn[u] = *reinterpret_cast<const uint4*>(kb + (size_t)jc * row_stride);
            vn[u] = *reinterpret_cast<const uint4*>(vb + (size_t)jc * row_stride);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int jj = j + u * KG;
            float kf[8], vf[8];
            unpack8(kk[u], kf);
            if (holds_new && jj == n - 1) {                                  // the key this workgroup has just rotated
#pragma unroll
                for (int e = 0; e < 8; ++e) kf[e] = s_knew[gl * 8 + e];
            }
            float sc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) sc += qv[e] * kf[e];
#pragma unroll
            for (int w = 1; w < G; w <<= 1) sc += __shfl_xor(sc, w, 64);    // the G lanes of a group are neighbours
            if (jj < j1) {                                                   // uniform inside a group
                unpack8(vv[u], vf);
                const float mn = fmaxf(m, sc);
                const float corr = __builtin_amdgcn_exp2f(m - mn), pw = __builtin_amdgcn_exp2f(sc - mn);
                l = l * corr + pw;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = acc[e] * corr + pw * vf[e];
                m = mn;
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) { kk[u] = kn[u]; vv[u] = vn[u]; }
    }
    // groups -> workgroup
    if (gl == 0) { s_m[grp] = m; s_l[grp] = l; }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[grp][gl * 8 + e] = acc[e];
    __syncthreads();
    if (tid < E) {
        float Mw = -INFINITY, Lw = 0.f, ow = 0.f;
        for (int g = 0; g < KG; ++g) Mw = fmaxf(Mw, s_m[g]);
        for (int g = 0; g < KG; ++g) {
            const float wgt = s_m[g] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s_m[g] - Mw);
            Lw += s_l[g] * wgt;
            ow += s_acc[g][tid] * wgt;
        }
        if (ns == 1) {
            reinterpret_cast<bf16_t*>(a.out)[(size_t)r * a.H * E + (size_t)h * E + tid] = f32_to_bf16(Lw > 0.f ? ow / Lw : 0.f);
        } else {
            // {max, sum, weighted V} of this share; the combine launch folds the shares
            float* mine = a.part + ((size_t)rh * kAttnMaxSplit + sp) * (E + 2);
            mine[2 + tid] = ow;
            if (tid == 0) { mine[0] = Mw; mine[1] = Lw; }
        }
    }
}

template <int E>
__global__ void __launch_bounds__(E) k_attn_combine(AttnArgs a) {
    constexpr int KG = 256 / (E / 8);
    const int tid = threadIdx.x, rh = blockIdx.x;
    const int h = rh % a.H, r = rh / a.H;
    const int b = r / a.T, s = r - b * a.T;
    int ns, per;
    split_of(visible_positions(a, b, s), a.NS, KG, ns, per);
    if (ns == 1) return;                                             // the main kernel has written this row already
    const float* base = a.part + (size_t)rh * kAttnMaxSplit * (E + 2);
    // every load of this kernel is issued before the first one is used: two memory round trips in all
    __shared__ float s_pm[kAttnMaxSplit], s_pl[kAttnMaxSplit];
    float ov[kAttnMaxSplit];
#pragma unroll
    for (int c = 0; c < kAttnMaxSplit; ++c) ov[c] = base[(size_t)(c < ns ? c : ns - 1) * (E + 2) + 2 + tid];
    if (tid < ns) { s_pm[tid] = base[(size_t)tid * (E + 2)]; s_pl[tid] = base[(size_t)tid * (E + 2) + 1]; }
    __syncthreads();
    float Mt = -INFINITY;
    for (int c = 0; c < ns; ++c) Mt = fmaxf(Mt, s_pm[c]);
    float Lt = 0.f, ot = 0.f;
#pragma unroll
    for (int c = 0; c < kAttnMaxSplit; ++c) {
        if (c < ns) {
            const float mc = s_pm[c];
            const float wgt = mc == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mc - Mt);
            Lt += s_pl[c] * wgt;
            ot += ov[c] * wgt;
        }
    }
    reinterpret_cast<bf16_t*>(a.out)[(size_t)r * a.H * E + (size_t)h * E + tid] = f32_to_bf16(Lt > 0.f ? ot / Lt : 0.f);
}

// ---- generic kernel: one workgroup per (row, head), positions in chunks through LDS ---------------
template <typename T, typename F>
__global__ void __launch_bounds__(256) k_attn_generic(AttnArgs a) {
    constexpr int CH = 512;
    __shared__ F s_w[CH];
    __shared__ F s_red[256];
    const int tid = threadIdx.x;
    const int h = blockIdx.x % a.H, r = blockIdx.x / a.H;
    const int b = r / a.T, s = r - b * a.T;
    long long nn = (long long)a.pos[b] + s + 1;
    const int n = (int)(nn < 0 ? 0 : (nn > a.S_max ? a.S_max : nn));
    const int E = a.E;
    const F* q = reinterpret_cast<const F*>(a.q_rot) + (size_t)r * a.H * E + (size_t)h * E;
    const T* kb = reinterpret_cast<const T*>(a.k_cache) + ((size_t)b * a.S_max * a.H + h) * E;
    const T* vb = reinterpret_cast<const T*>(a.v_cache) + ((size_t)b * a.S_max * a.H + h) * E;
    const size_t row_stride = (size_t)a.H * E;
    T* orow = reinterpret_cast<T*>(a.out) + (size_t)r * a.H * E + (size_t)h * E;
    F m_run = -INFINITY, l_run = 0;
    F acc[4] = {0, 0, 0, 0};                      // output elements tid, tid + 256, ... (E <= 1024)
    for (int c0 = 0; c0 < n; c0 += CH) {
        const int cn = n - c0 < CH ? n - c0 : CH;
        F cmax = -INFINITY;
        for (int j = tid; j < cn; j += 256) {
            const T* kj = kb + (size_t)(c0 + j) * row_stride;
            F sc = 0;
            for (int e = 0; e < E; ++e) sc += q[e] * (F)AIo<T>::ld(kj + e);
            sc *= (F)a.scale;
            s_w[j] = sc;
            cmax = sc > cmax ? sc : cmax;
        }
        s_red[tid] = cmax;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) { if (tid < w) s_red[tid] = s_red[tid] > s_red[tid + w] ? s_red[tid] : s_red[tid + w]; __syncthreads(); }
        const F m_new = s_red[0] > m_run ? s_red[0] : m_run;
        __syncthreads();
        F part = 0;
        for (int j = tid; j < cn; j += 256) { const F w = exp(s_w[j] - m_new); s_w[j] = w; part += w; }
        s_red[tid] = part;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) { if (tid < w) s_red[tid] += s_red[tid + w]; __syncthreads(); }
        const F corr = m_run == -INFINITY ? (F)0 : exp(m_run - m_new);
        l_run = l_run * corr + s_red[0];
        for (int i = 0; i < 4; ++i) {
            const int e = tid + 256 * i;
            if (e < E) {
                F o = acc[i] * corr;
                for (int j = 0; j < cn; ++j) o += s_w[j] * (F)AIo<T>::ld(vb + (size_t)(c0 + j) * row_stride + e);
                acc[i] = o;
            }
        }
        m_run = m_new;
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        const int e = tid + 256 * i;
        if (e < E) orow[e] = AIo<T>::cvt((double)(l_run > 0 ? acc[i] / l_run : (F)0));
    }
}

int attn_decode(const void* q, const lr_kv_target* kv, void* out, float scale, float rope_base, int dtype,
                bool fast, void* ws, hipStream_t s) {
    const int64_t M = kv->B * kv->tokens_per_seq, H = kv->n_heads, E = kv->head_dim, d = H * E;
    const AttnLayout L = attn_layout(ws, M, d, H);
    AttnArgs a;
    a.q = q; a.q_rot = L.q_rot; a.k_cache = kv->k_cache; a.v_cache = kv->v_cache; a.pos = kv->pos; a.out = out;
    a.part = L.part;
    a.M = (int)M; a.T = (int)kv->tokens_per_seq; a.H = (int)H; a.E = (int)E; a.S_max = (int)kv->S_max;
    a.scale = scale; a.rope_base = (double)rope_base;
    const long long pairs = (long long)M * H * (E / 2);
    const unsigned pg = (unsigned)((pairs + 255) / 256 < 4096 ? (pairs + 255) / 256 : 4096);
    if (fast) {
        // about two workgroups per CU, at most kAttnMaxSplit per (row, head)
        int ns = (int)((512 + M * H - 1) / (M * H));
        a.NS = ns < 1 ? 1 : (ns > kAttnMaxSplit ? kAttnMaxSplit : ns);
        a.qscale = scale * 1.4426950408889634f;
        const bool fused = kv->tokens_per_seq == 1;
        if (!fused) hipLaunchKernelGGL((k_attn_prepare<bf16_t, float>), dim3(pg), dim3(256), 0, s, a);
        const dim3 grid((unsigned)(M * H * a.NS)), cgrid((unsigned)(M * H));
#define LR_ATTN_LAUNCH(EE)                                                                                  \
        do {                                                                                                \
            if (fused) hipLaunchKernelGGL((k_attn_decode<EE, true>), grid, dim3(256), 0, s, a);             \
            else hipLaunchKernelGGL((k_attn_decode<EE, false>), grid, dim3(256), 0, s, a);                  \
            if (a.NS > 1) hipLaunchKernelGGL((k_attn_combine<EE>), cgrid, dim3(EE), 0, s, a);               \
        } while (0)
        if (E == 64) LR_ATTN_LAUNCH(64);
        else if (E == 128) LR_ATTN_LAUNCH(128);
        else LR_ATTN_LAUNCH(256);
#undef LR_ATTN_LAUNCH
        return launch_status("decode attention");
    }
    a.NS = 1; a.qscale = 1.f;
    const dim3 grid((unsigned)(M * H));
    if (dtype == LR_BF16) {
        hipLaunchKernelGGL((k_attn_prepare<bf16_t, float>), dim3(pg), dim3(256), 0, s, a);
        hipLaunchKernelGGL((k_attn_generic<bf16_t, float>), grid, dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL((k_attn_prepare<float, double>), dim3(pg), dim3(256), 0, s, a);
        hipLaunchKernelGGL((k_attn_generic<float, double>), grid, dim3(256), 0, s, a);
    }
    return launch_status("decode attention (generic)");
}

}  // namespace lr
