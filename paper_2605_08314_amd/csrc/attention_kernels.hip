// Decode attention over the dense KV cache this library writes (paper Section 3.1, decode-attention
// paragraph: the present token's q/k/v are reconstructed once, the history is read from a standard
// dense cache [batch, position, head, head_dim]; Section 4: RoPE on q and k).
//
// Two launches per call:
//   k_attn_prepare   rotates the T new key rows of every sequence in place in the cache and writes the
//                    rotated queries (pre-scaled for the fast kernel) to the workspace;
//   k_attn_decode    one workgroup per (token row, head, split of the visible positions): streams its
//                    share of K and V once (the step is bound by those bytes), online softmax per group
//                    of E/8 lanes, groups combined through LDS, splits combined by the last workgroup
//                    to arrive (partials and the arrival counter go through device-coherent accesses).
// A generic kernel (any head_dim, fp32 caches, fp64 arithmetic for fp32 data) covers what the fast one
// does not.
#include "attention.hpp"

namespace lr {

size_t attn_ws_bytes(int64_t M, int64_t d, int64_t H) {
    const int64_t E = H > 0 ? d / H : 0;
    return kHeaderBytes + align256((size_t)M * (size_t)d * 8) +
           align256((size_t)M * (size_t)H * kAttnMaxSplit * (size_t)(E + 2) * 4) + align256((size_t)M * (size_t)H * 4);
}

AttnLayout attn_layout(void* ws, int64_t M, int64_t d, int64_t H) {
    const int64_t E = H > 0 ? d / H : 0;
    AttnLayout L;
    char* p = (char*)ws + kHeaderBytes;
    L.q_rot = p; p += align256((size_t)M * (size_t)d * 8);
    L.part = (float*)p; p += align256((size_t)M * (size_t)H * kAttnMaxSplit * (size_t)(E + 2) * 4);
    L.counter = (uint32_t*)p;
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
    float* part; uint32_t* counter;
    int M, T, H, E, S_max, NS;
    float qscale;           // what the stored queries are multiplied by (fast path: scale * log2 e; generic: 1)
    float scale;
    double rope_base;       // <= 0: no rotation
};

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
            const double ang = (double)p * pow(a.rope_base, -2.0 * (double)i / (double)a.E);
            const double c = cos(ang), sn = sin(ang);
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
__device__ __forceinline__ uint2 ld_dev64(const void* p) {
    const uint64_t v = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
__device__ __forceinline__ void st_dev64(void* p, float lo, float hi) {
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), (uint64_t)__float_as_uint(lo) | ((uint64_t)__float_as_uint(hi) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

template <int E>
__global__ void __launch_bounds__(256) k_attn_decode(AttnArgs a) {
    constexpr int G = E / 8;            // lanes that share one cached position (16 bytes each)
    constexpr int KG = 256 / G;         // positions a workgroup takes per sweep = number of lane groups
    constexpr int UNR = 4;              // positions in flight per group
    __shared__ float s_m[KG], s_l[KG];
    __shared__ float s_acc[KG][E];
    __shared__ uint32_t s_last;
    const int tid = threadIdx.x, grp = tid / G, gl = tid % G;
    const int sp = blockIdx.x % a.NS, rh = blockIdx.x / a.NS;
    const int h = rh % a.H, r = rh / a.H;
    const int b = r / a.T, s = r - b * a.T;
    long long nn = (long long)a.pos[b] + s + 1;                 // visible positions (causal)
    const int n = (int)(nn < 0 ? 0 : (nn > a.S_max ? a.S_max : nn));
    int per = (n + a.NS - 1) / a.NS;
    per = (per + KG - 1) / KG * KG;
    const int j0 = sp * per, j1 = (j0 + per < n) ? j0 + per : n;

    float qv[8];
    {
        const float* q = reinterpret_cast<const float*>(a.q_rot) + (size_t)r * a.H * E + (size_t)h * E + gl * 8;
        const float4 q0 = *reinterpret_cast<const float4*>(q), q1 = *reinterpret_cast<const float4*>(q + 4);
        qv[0] = q0.x; qv[1] = q0.y; qv[2] = q0.z; qv[3] = q0.w; qv[4] = q1.x; qv[5] = q1.y; qv[6] = q1.z; qv[7] = q1.w;
    }
    const size_t row_stride = (size_t)a.H * E;
    const bf16_t* kb = reinterpret_cast<const bf16_t*>(a.k_cache) + ((size_t)b * a.S_max * a.H + h) * E + gl * 8;
    const bf16_t* vb = reinterpret_cast<const bf16_t*>(a.v_cache) + ((size_t)b * a.S_max * a.H + h) * E + gl * 8;

    float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int j = j0 + grp; j < j1; j += KG * UNR) {
        uint4 kk[UNR], vv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int jj = j + u * KG;
            const int jc = jj < j1 ? jj : j;                    // positions past the end repeat a valid one; unused
            kk[u] = *reinterpret_cast<const uint4*>(kb + (size_t)jc * row_stride);
            vv[u] = *reinterpret_cast<const uint4*>(vb + (size_t)jc * row_stride);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            float kf[8], vf[8];
            unpack8(kk[u], kf);
            float sc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) sc += qv[e] * kf[e];
#pragma unroll
            for (int w = 1; w < G; w <<= 1) sc += __shfl_xor(sc, w, 64);    // the G lanes of a group are neighbours
            if (j + u * KG < j1) {                                          // uniform inside a group
                unpack8(vv[u], vf);
                const float mn = fmaxf(m, sc);
                const float corr = __builtin_amdgcn_exp2f(m - mn), pw = __builtin_amdgcn_exp2f(sc - mn);
                l = l * corr + pw;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = acc[e] * corr + pw * vf[e];
                m = mn;
            }
        }
    }
    // groups -> workgroup
    if (gl == 0) { s_m[grp] = m; s_l[grp] = l; }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[grp][gl * 8 + e] = acc[e];
    __syncthreads();
    float Mw = -INFINITY, Lw = 0.f, ow = 0.f;
    if (tid < E) {
        for (int g = 0; g < KG; ++g) Mw = fmaxf(Mw, s_m[g]);
        for (int g = 0; g < KG; ++g) {
            const float wgt = s_m[g] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s_m[g] - Mw);
            Lw += s_l[g] * wgt;
            ow += s_acc[g][tid] * wgt;
        }
    }
    bf16_t* orow = reinterpret_cast<bf16_t*>(a.out) + (size_t)r * a.H * E + (size_t)h * E;
    if (a.NS == 1) {
        if (tid < E) orow[tid] = f32_to_bf16(Lw > 0.f ? ow / Lw : 0.f);
        return;
    }
    // splits -> result: hand {max, sum, weighted V} to whoever arrives last
    float* mine = a.part + ((size_t)rh * kAttnMaxSplit + sp) * (E + 2);
    const float o1 = __shfl_down(ow, 1, 64);                        // every lane takes part; even lanes store a pair
    if (tid < E && (tid & 1) == 0) st_dev64(mine + 2 + tid, ow, o1);
    if (tid == 0) st_dev64(mine, Mw, Lw);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");          // this wave's stores have been performed
    __syncthreads();
    if (tid == 0) {
        const uint32_t old = __hip_atomic_fetch_add(a.counter + rh, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (old == (uint32_t)a.NS - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    if (tid < E) {
        const float* base = a.part + (size_t)rh * kAttnMaxSplit * (E + 2);
        float Mt = -INFINITY;
        for (int c = 0; c < a.NS; ++c) Mt = fmaxf(Mt, __uint_as_float(ld_dev64(base + (size_t)c * (E + 2)).x));
        float Lt = 0.f, ot = 0.f;
        for (int c = 0; c < a.NS; ++c) {
            const uint2 ml = ld_dev64(base + (size_t)c * (E + 2));
            const float mc = __uint_as_float(ml.x);
            const float wgt = mc == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mc - Mt);
            const uint2 ov = ld_dev64(base + (size_t)c * (E + 2) + 2 + (tid & ~1));
            Lt += __uint_as_float(ml.y) * wgt;
            ot += __uint_as_float((tid & 1) ? ov.y : ov.x) * wgt;
        }
        orow[tid] = f32_to_bf16(Lt > 0.f ? ot / Lt : 0.f);
    }
    if (tid == 0) __hip_atomic_store(a.counter + rh, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
    a.part = L.part; a.counter = L.counter;
    a.M = (int)M; a.T = (int)kv->tokens_per_seq; a.H = (int)H; a.E = (int)E; a.S_max = (int)kv->S_max;
    a.scale = scale; a.rope_base = (double)rope_base;
    const long long pairs = (long long)M * H * (E / 2);
    const unsigned pg = (unsigned)((pairs + 255) / 256 < 4096 ? (pairs + 255) / 256 : 4096);
    if (fast) {
        // enough workgroups to cover the chip three times over, at most kAttnMaxSplit per (row, head)
        int ns = (int)((768 + M * H - 1) / (M * H));
        a.NS = ns < 1 ? 1 : (ns > kAttnMaxSplit ? kAttnMaxSplit : ns);
        a.qscale = scale * 1.4426950408889634f;
        hipLaunchKernelGGL((k_attn_prepare<bf16_t, float>), dim3(pg), dim3(256), 0, s, a);
        const dim3 grid((unsigned)(M * H * a.NS));
        if (E == 64) hipLaunchKernelGGL((k_attn_decode<64>), grid, dim3(256), 0, s, a);
        else if (E == 128) hipLaunchKernelGGL((k_attn_decode<128>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((k_attn_decode<256>), grid, dim3(256), 0, s, a);
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
