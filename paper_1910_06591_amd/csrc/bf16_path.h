// bf16 (matrix-core) path: host-side weight packing, device state, support
// check and the per-step kernel sequence.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <string>
#include <vector>

#include "plan.h"
#include "kernels_fp32.h"
#include "gemm_bf16.h"
#include "gemm_bf16_lds.h"
#include "conv_stack_bf16.h"
#include "conv_stack_fused.h"
#include "resnet_fused.h"
#include "resnet_layerwise.h"
#include "resnet_blockfused.h"
#include "resnet_firstpool.h"
#include "resnet_convpool.h"
#include "resnet_convtile.h"

namespace seedinf {

// ---- the deep-ResNet torsos this build has fused kernels for ----------------
// DMLab-shaped: 72x96x3 frames, sections 16/32/32.
using DmS1 = SecCfg<72, 96, 3, 16, IN_U8_C3, 4, 36>;
using DmS2 = SecCfg<36, 48, 16, 32, IN_LDS, 8, 0, 8, 2, 0>;     // pooled map 18 x 24 with a 28-cell pitch (TileMap1824)
using DmS3 = SecCfg<18, 24, 32, 32, IN_LDS, 4, 0, 8, 0, 2>;
// Football-shaped: 72x96x16 minimap planes, sections 16/32/32/32.
using FbS1 = SecCfg<72, 96, 16, 16, IN_U8_PLANAR, 4, 8>;
using FbS4 = SecCfg<9, 12, 32, 32, IN_LDS, 5, 0, 2>;

enum { TORSO_NONE = 0, TORSO_DMLAB = 1, TORSO_FOOTBALL = 2 };

// The conv stack this build has a fused kernel for: the recurrent Atari agent's (Appendix A.3.1), with four
// stacked frames or one.
inline bool match_r2d2_stack(const seed_arch_t& a)
{
    return a.torso == SEED_TORSO_CONV_STACK && a.obs_h == 84 && a.obs_w == 84 && (a.obs_c == 4 || a.obs_c == 1) && a.n_conv == 3 &&
           a.conv_ch[0] == 32 && a.conv_k[0] == 8 && a.conv_stride[0] == 4 &&
           a.conv_ch[1] == 64 && a.conv_k[1] == 4 && a.conv_stride[1] == 2 &&
           a.conv_ch[2] == 64 && a.conv_k[2] == 3 && a.conv_stride[2] == 1;
}

inline int match_resnet(const seed_arch_t& a)
{
    if (a.torso != SEED_TORSO_RESNET || a.obs_h != 72 || a.obs_w != 96) return TORSO_NONE;
    if (a.obs_c == 3 && a.n_sections == 3 && a.section_ch[0] == 16 && a.section_ch[1] == 32 && a.section_ch[2] == 32)
        return TORSO_DMLAB;
    if (a.obs_c == 16 && a.n_sections == 4 && a.section_ch[0] == 16 && a.section_ch[1] == 32 &&
        a.section_ch[2] == 32 && a.section_ch[3] == 32)
        return TORSO_FOOTBALL;
    return TORSO_NONE;
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

inline seed_status_t bf16_supported(const Plan& p, std::string& err)
{
    const seed_arch_t& a = p.arch;
    auto no = [&](const char* m) { err = std::string("bf16 mode: ") + m + " (fp32 mode supports every valid arch)"; return SEED_ERR_UNSUPPORTED_ARCH; };
    if (a.torso == SEED_TORSO_RESNET) {
        // shapes without a fused kernel run layer by layer; that path needs whole 16-channel tiles
        if (match_resnet(a) == TORSO_NONE)
            for (int i = 0; i < a.n_sections; ++i)
                if (a.section_ch[i] % 16) return no("ResNet section channels must be multiples of 16");
    } else if (!match_r2d2_stack(a)) {
        for (size_t l = 0; l < p.convs.size(); ++l) {
            const ConvLayer& c = p.convs[l];
            if (c.Cout % 16) return no("conv channels must be multiples of 16");
            if ((c.k * c.Cin) % 8 || (c.k * c.k * c.Cin) % 32) return no("conv k*Cin must be a multiple of 8 and k*k*Cin of 32");
            if ((c.W * c.Cin) % 8 || (c.stride * c.Cin) % 8 || ((size_t)c.H * c.W * c.Cin) % 8) return no("conv rows must be 8-element aligned");
        }
        if (p.flat % 32) return no("the conv stack's flattened output must be a multiple of 32 values");
    }   // (the fused conv stack has none of these limits)
    if (a.lstm_units % 16) return no("lstm_units must be a multiple of 16");
    if (a.head == SEED_HEAD_DUELING_Q && a.head_hidden % 16) return no("head_hidden must be a multiple of 16");
    return SEED_OK;
}

// ---- packing plan --------------------------------------------------------------
// The packed operand stream of a network depends on the weights only through a gather: every 16-bit element of it
// is zero padding, the bf16 rounding of one canonical weight, or one half of a canonical fp32 bias.  The host
// works that gather out ONCE per handle (the layouts below, run over a vector that holds each weight's own index)
// and uploads it as a table; the device then packs any weight vector with one kernel (bf16_repack_kernel), at
// creation and at every weight update, so an update costs the host one copy of the flat vector.
//   table entry = 4 * (index + 1) + kind;  kind 1: bf16(w[index]), 2 / 3: low / high half of the fp32 w[index];
//   0 = zero.  The fp32 bias table holds index + 1, or 0 for padding.
enum { PK_ZERO = 0, PK_BF16 = 1, PK_F32_LO = 2, PK_F32_HI = 3 };
inline uint32_t pk_entry(float index_plus_1, int kind)
{
    return index_plus_1 == 0.f ? 0u : (((uint32_t)index_plus_1) << 2) | (uint32_t)kind;
}

// A-operand fragments [ftile][kchunk][lane][8] from value(f, k) (value = the weight's index + 1, or 0)
template <class F>
inline void pack_a(std::vector<uint32_t>& out, int n_ftiles, int kchunks, F value)
{
    size_t base = out.size();
    out.resize(base + (size_t)n_ftiles * kchunks * 64 * 8);
    uint32_t* d = out.data() + base;
    for (int ft = 0; ft < n_ftiles; ++ft)
        for (int kc = 0; kc < kchunks; ++kc)
            for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 8; ++e)
                    *d++ = pk_entry(value(ft * 16 + (lane & 15), kc * 32 + 8 * (lane >> 4) + e), PK_BF16);
}

struct ConvStackLayerDev { size_t wp_off; size_t koff_off; int kchunks; };
// layer-by-layer ResNet, one 3x3 convolution; first_off: the network's first layer packed for the fused
// convolution + pooling kernel as well (LW_NONE: not packed that way)
constexpr size_t LW_NONE = (size_t)-1;
struct LwLayerDev { size_t wp_off; size_t ktab_off; int kchunks; size_t first_off = LW_NONE; };
inline bool first_pool_supported(const ConvLayer& c)
{
    return (c.Cin <= 4 || c.Cin == 8 || c.Cin == 16) && (c.Cout == 16 || c.Cout == 32 || c.Cout == 64);
}

// Device pointers into one uploaded copy of the packed weights.
struct Bf16WeightSet {
    const bf16x8* wp_fc = nullptr; const float* bias_fc = nullptr;
    const bf16x8* wp_lstm = nullptr;
    const bf16x8* wp_hid = nullptr; const float* bias_hid = nullptr;
    const bf16x8* wp_conv = nullptr;
    SecWeights sec[4];
};

// Host-side result of packing one set of weights; the offsets depend on the arch only.
struct Bf16Packed {
    std::vector<uint32_t> pk;                  // gather table of the packed 16-bit operand stream (see pk_entry)
    std::vector<uint32_t> fb;                  // gather table of the padded fp32 biases: index + 1, 0 = zero
    std::vector<int> ko;                       // conv-stack offset tables (weight-independent)
    size_t sec_off[4][5] = {};
    size_t off_fc = 0, off_bfc = 0, off_lstm = 0, off_hid = 0, off_bhid = 0;
    std::vector<ConvStackLayerDev> stack;
    std::vector<LwLayerDev> lw;                // per section: conv0, block1.a, block1.b, block2.a, block2.b
    int kc_fc = 0, ft_fc = 0, kc1_lstm = 0, ft_hid = 0;
};

struct Bf16State {
    int torso_kind = TORSO_NONE;
    bool stack_fused = false;                  // conv stack with the fused kernel
    int n_cu = 256;
    char* arena = nullptr;
    // two copies of the packed weights: steps read ws[active]; a weight update fills the other and flips
    Bf16WeightSet ws[2];
    int active = 0;
    size_t o_pk[2] = {0, 0}, o_fb[2] = {0, 0};
    size_t pk_bytes = 0, fb_bytes = 0;
    const uint32_t* tab_pk = nullptr; const uint32_t* tab_fb = nullptr;   // device: the packing plan's gather tables
    int kc_fc = 0, ft_fc = 0, kc1_lstm = 0, ft_hid = 0;
    std::vector<ConvStackLayerDev> stack;
    std::vector<LwLayerDev> lw;
    const int* koff = nullptr;
    // layer-by-layer ResNet workspace: conv0 output at input resolution; R / U conv inputs; x residual stream
    __bf16* lw_c0 = nullptr; __bf16* lw_r = nullptr; __bf16* lw_u = nullptr; float* lw_x = nullptr;
    // activations
    __bf16* act[2] = {nullptr, nullptr};
    __bf16* feat = nullptr; int ldf = 0;
    __bf16* fc_bf16 = nullptr; int ldfc = 0;
    float* fc_f32 = nullptr;
};

inline void bf16_destroy(Bf16State* s)
{
    if (!s) return;
    if (s->arena) (void)hipFree(s->arena);
    delete s;
}

#define BF_TRY(expr)                                                             \
    do {                                                                         \
        hipError_t e_ = (expr);                                                  \
        if (e_ != hipSuccess) {                                                  \
            err = std::string(#expr) + ": " + hipGetErrorString(e_);             \
            return e_ == hipErrorOutOfMemory ? SEED_ERR_OOM : SEED_ERR_DEVICE;   \
        }                                                                        \
    } while (0)

// weight of output channel f at packed K index k (chunk k/32, lane group (k%32)/8, element k%8) of a 3x3
// convolution with CIN input channels, following the kernels' K layout (KMap)
template <int CIN>
inline float planar_weight(const float* w, int cout, int f, int k)
{
    const int kc = k / 32, g = (k % 32) / 8, e = k % 8;
    const int tap = KMap<CIN>::tap(kc, g);
    if (tap < 0 || tap > 8) return 0.f;
    const int ch = KMap<CIN>::cg(kc, g) * 8 + e;
    return w[((size_t)tap * CIN + ch) * cout + f];
}

// one 1 KiB chunk after a layer's fragments: its first C floats are the layer's biases
inline void pack_bias_chunk(std::vector<uint32_t>& pk, const float* bias, int C)
{
    size_t base = pk.size();
    pk.resize(base + 512, 0);
    for (int c = 0; c < C; ++c) {
        pk[base + 2 * c] = pk_entry(bias[c], PK_F32_LO);
        pk[base + 2 * c + 1] = pk_entry(bias[c], PK_F32_HI);
    }
}

template <class S>
inline void pack_section(std::vector<uint32_t>& pk, const float* w, const Section& sec, size_t (&off)[5])
{
    const ConvLayer& c0 = sec.conv0;
    const float* w0 = w + c0.w_off;
    off[0] = pk.size();
    if constexpr (S::INKIND == IN_U8_C3) {
        // four fragments (see conv0_pool3): lane group g -> buffer row g/2 of a row pair, pixel pair g%2; element e ->
        // pixel e/4, channel e%4.  Fragment 0: kernel rows (0 | 1), 1: (2 | none), 2: (none | 0), 3: (1 | 2).
        pack_a(pk, S::FT, 4, [&](int f, int k) -> float {
            const int fr = k / 32, g = (k % 32) / 8, e = k % 8;
            const int half = g >> 1;
            const int kh = fr == 0 ? half : (fr == 1 ? (half ? -1 : 2) : (fr == 2 ? (half ? 0 : -1) : 1 + half));
            const int kw = 2 * (g & 1) + e / 4, ch = e % 4;
            if (kh < 0 || kw > 2 || ch > 2) return 0.f;
            return w0[((size_t)(kh * 3 + kw) * 3 + ch) * S::C + f];
        });
    } else {
        pack_a(pk, S::FT, S::KC0, [&](int f, int k) -> float { return planar_weight<S::CIN>(w0, S::C, f, k); });
    }
    pack_bias_chunk(pk, w + c0.b_off, S::C);
    for (int j = 0; j < 4; ++j) {
        const float* wb = w + sec.block[j].w_off;
        off[1 + j] = pk.size();
        if constexpr (S::SLIDE) {
            // sliding-window layout: chunk = weight fragment, lane group -> (tap, channel group) per SlideMap16
            pack_a(pk, 1, SlideMap16::NFRAG, [&](int f, int k) -> float {
                const int fr = k / 32, g = (k % 32) / 8, e = k % 8;
                const int tap = SlideMap16::tap(fr, g);
                if (tap < 0) return 0.f;
                return wb[((size_t)tap * S::C + SlideMap16::cg(g) * 8 + e) * S::C + f];
            });
        } else {
            pack_a(pk, S::FT, S::KCB, [&](int f, int k) -> float { return planar_weight<S::C>(wb, S::C, f, k); });
        }
        pack_bias_chunk(pk, w + sec.block[j].b_off, S::C);
    }
}

// Lays out every layer's operands for the bf16 kernels as gather tables over the canonical flat weight vector
// (host side, once per handle).
inline void bf16_pack(const Plan& p, int torso_kind, int ldf_, int ldfc_, Bf16Packed& o)
{
    const seed_arch_t& a = p.arch;
    // the layouts below read "weights"; here every weight is its own index + 1 (exact in fp32 up to 2^24)
    std::vector<float> iota(p.n_weights);
    for (size_t i = 0; i < iota.size(); ++i) iota[i] = (float)(i + 1);
    const float* w = iota.data();
    std::vector<uint32_t>& pk = o.pk;
    std::vector<float> fb;
    std::vector<int>& ko = o.ko;
    size_t (&sec_off)[4][5] = o.sec_off;
    if (a.torso == SEED_TORSO_RESNET && torso_kind == TORSO_NONE) {
        auto pack_conv = [&](const ConvLayer& c, bool first) {
            LwLayerDev d;
            const int K = 9 * c.Cin;
            d.kchunks = (K + 31) / 32;
            d.wp_off = pk.size();
            const float* wl = w + c.w_off;
            pack_a(pk, c.Cout / 16, d.kchunks, [&](int f, int k) -> float { return k < K ? wl[(size_t)k * c.Cout + f] : 0.f; });
            if (ko.size() & 1) ko.push_back(0);            // the table is read as int2
            d.ktab_off = ko.size();
            for (int kc = 0; kc < d.kchunks; ++kc)
                for (int g = 0; g < 4; ++g) {
                    const int k0 = kc * 32 + g * 8;
                    if (k0 >= K || (c.Cin & 7)) { ko.push_back(0); ko.push_back(-1); continue; }
                    const int tap = k0 / c.Cin, dy = tap / 3 - 1, dx = tap % 3 - 1;
                    ko.push_back((dy * c.W + dx) * c.Cin + k0 % c.Cin);
                    ko.push_back((dy + 1) | ((dx + 1) << 8));
                }
            if (first && first_pool_supported(c)) d.first_off = d.wp_off;       // 8 or 16 planes: the same packing
            if (first && first_pool_supported(c) && c.Cin <= 4) {
                d.first_off = pk.size();
                pack_a(pk, c.Cout / 16, 2, [&](int f, int k) -> float {
                    int dy, dx, ci;
                    first_pool_k(k, dy, dx, ci);
                    return dy < 3 && dx < 3 && ci < c.Cin ? wl[(size_t)((dy * 3 + dx) * c.Cin + ci) * c.Cout + f] : 0.f;
                });
            }
            o.lw.push_back(d);
        };
        for (size_t si = 0; si < p.sections.size(); ++si) {
            const Section& sec = p.sections[si];
            pack_conv(sec.conv0, si == 0);
            for (int j = 0; j < 4; ++j) pack_conv(sec.block[j], false);
        }
    } else if (a.torso == SEED_TORSO_RESNET) {
        if (torso_kind == TORSO_DMLAB) {
            pack_section<DmS1>(pk, w, p.sections[0], sec_off[0]);
            pack_section<DmS2>(pk, w, p.sections[1], sec_off[1]);
            pack_section<DmS3>(pk, w, p.sections[2], sec_off[2]);
        } else {
            pack_section<FbS1>(pk, w, p.sections[0], sec_off[0]);
            pack_section<DmS2>(pk, w, p.sections[1], sec_off[1]);
            pack_section<DmS3>(pk, w, p.sections[2], sec_off[2]);
            pack_section<FbS4>(pk, w, p.sections[3], sec_off[3]);
        }
    } else {
        for (const ConvLayer& c : p.convs) {
            ConvStackLayerDev d;
            const int K = c.k * c.k * c.Cin;
            d.kchunks = K / 32;
            d.wp_off = pk.size();
            const float* wl = w + c.w_off;
            pack_a(pk, c.Cout / 16, d.kchunks, [&](int f, int k) -> float { return wl[(size_t)k * c.Cout + f]; });
            d.koff_off = ko.size();
            for (int kc = 0; kc < d.kchunks; ++kc)
                for (int g = 0; g < 4; ++g) {
                    int k0 = kc * 32 + g * 8;
                    int kh = k0 / (c.k * c.Cin), rem = k0 % (c.k * c.Cin);
                    ko.push_back(kh * c.W * c.Cin + rem);
                }
            o.stack.push_back(d);
        }
    }
    // linear layer: K = ldf (zero rows past flat), features padded to whole tiles
    const int F = a.fc_units;
    o.ft_fc = (F + 15) / 16;
    o.kc_fc = ldf_ / 32;
    o.off_fc = pk.size();
    {
        const float* wf = w + p.fc_w;
        const int flat = (int)p.flat;
        pack_a(pk, o.ft_fc, o.kc_fc, [&](int f, int k) -> float { return (k < flat && f < F) ? wf[(size_t)k * F + f] : 0.f; });
    }
    o.off_bfc = fb.size();
    for (int f = 0; f < o.ft_fc * 16; ++f) fb.push_back(f < F ? w[p.fc_b + f] : 0.f);
    // LSTM: K = [ldfc feature columns | h columns]; feature tile (ut, gate)
    const int Hn = a.lstm_units;
    if (Hn > 0) {
        o.off_lstm = pk.size();
        o.kc1_lstm = ldfc_ / 32;
        const int kc2 = (Hn + 31) / 32;
        const float* wl = w + p.lstm_w;
        const int G4 = 4 * Hn, ldfc = ldfc_, A = a.num_actions;
        pack_a(pk, (Hn / 16) * 4, o.kc1_lstm + kc2, [&](int f, int k) -> float {
            int ft = f / 16, m = f % 16;
            int col = (ft % 4) * Hn + (ft / 4) * 16 + m;
            if (k < ldfc) return k < F ? wl[(size_t)k * G4 + col] : 0.f;
            int hk = k - ldfc;
            return hk < Hn ? wl[(size_t)(F + A + 1 + hk) * G4 + col] : 0.f;
        });
    }
    // dueling hidden layers: features [value stream | advantage stream]
    if (a.head == SEED_HEAD_DUELING_Q) {
        const int hid = a.head_hidden, core = p.core;
        const int kc = Hn > 0 ? (core + 31) / 32 : ldfc_ / 32;
        o.ft_hid = 2 * hid / 16;
        o.off_hid = pk.size();
        const float* wv = w + p.v1_w;
        const float* wa = w + p.a1_w;
        pack_a(pk, o.ft_hid, kc, [&](int f, int k) -> float {
            if (k >= core) return 0.f;
            return f < hid ? wv[(size_t)k * hid + f] : wa[(size_t)k * hid + (f - hid)];
        });
        o.off_bhid = fb.size();
        for (int f = 0; f < hid; ++f) fb.push_back(w[p.v1_b + f]);
        for (int f = 0; f < hid; ++f) fb.push_back(w[p.a1_b + f]);
    }
    o.fb.resize(fb.size());
    for (size_t i = 0; i < fb.size(); ++i) o.fb[i] = (uint32_t)fb[i];
}

// The device side of the packing plan: one thread per 16-bit element of the operand stream (and per bias).
// fp32 -> bf16 rounds to nearest even; a NaN stays a NaN.
__global__ __launch_bounds__(256) void bf16_repack_kernel(const float* __restrict__ w, const uint32_t* __restrict__ tab_pk,
                                                          size_t n_pk, uint16_t* __restrict__ pk,
                                                          const uint32_t* __restrict__ tab_fb, size_t n_fb, float* __restrict__ fb)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_pk + n_fb; i += stride) {
        if (i < n_pk) {
            const uint32_t e = tab_pk[i];
            uint16_t v = 0;
            if (e) {
                uint32_t u = __float_as_uint(w[(e >> 2) - 1]);
                const uint32_t kind = e & 3u;
                if (kind == PK_BF16) {
                    if ((u & 0x7fffffffu) > 0x7f800000u) u = (u >> 16) | 0x40u;
                    else u = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
                } else if (kind == PK_F32_HI) {
                    u >>= 16;
                }
                v = (uint16_t)(u & 0xffffu);
            }
            pk[i] = v;
        } else {
            const uint32_t e = tab_fb[i - n_pk];
            fb[i - n_pk] = e ? w[e - 1] : 0.f;
        }
    }
}

// Resolves the pointers of weight set `set` from the packing offsets.
inline void bf16_bind(Bf16State* s, const Plan& p, const Bf16Packed& o, int set)
{
    const seed_arch_t& a = p.arch;
    Bf16WeightSet& W = s->ws[set];
    const uint16_t* dpk = (const uint16_t*)(s->arena + s->o_pk[set]);
    auto frag = [&](size_t off) { return (const bf16x8*)(dpk + off); };
    const float* dfb = (const float*)(s->arena + s->o_fb[set]);
    W.wp_fc = frag(o.off_fc); W.bias_fc = dfb + o.off_bfc;
    if (a.lstm_units > 0) W.wp_lstm = frag(o.off_lstm);
    if (a.head == SEED_HEAD_DUELING_Q) { W.wp_hid = frag(o.off_hid); W.bias_hid = dfb + o.off_bhid; }
    W.wp_conv = frag(0);
    if (a.torso == SEED_TORSO_RESNET && s->torso_kind != TORSO_NONE) {
        for (size_t si = 0; si < p.sections.size(); ++si) {
            SecWeights& sw = W.sec[si];
            sw.w0 = frag(o.sec_off[si][0]);
            for (int j = 0; j < 4; ++j) sw.wb[j] = frag(o.sec_off[si][1 + j]);
        }
    }
}

// Packs the canonical weights at d_w (device) into weight set `set` of the arena, on stream st.
inline void bf16_repack(Bf16State* s, const float* d_w, int set, hipStream_t st)
{
    const size_t n_pk = s->pk_bytes / 2, n_fb = s->fb_bytes / 4;
    const size_t n = n_pk + n_fb;
    if (n == 0) return;
    const size_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(bf16_repack_kernel, dim3((unsigned)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, st, d_w, s->tab_pk, n_pk,
                       (uint16_t*)(s->arena + s->o_pk[set]), s->tab_fb, n_fb, (float*)(s->arena + s->o_fb[set]));
}

// d_w: the canonical weights, already on the device (set 0 is packed from them here).
inline seed_status_t bf16_create(const Plan& p, const float* d_w, Bf16State** out, std::string& err)
{
    const seed_arch_t& a = p.arch;
    Bf16State* s = new Bf16State;
    *out = s;                                  // owned by the handle from here on (freed on any failure by the caller)
    int dev = 0;
    BF_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    BF_TRY(hipGetDeviceProperties(&prop, dev));
    s->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    s->torso_kind = match_resnet(a);
    s->stack_fused = match_r2d2_stack(a);
    s->ldf = round_up((int)p.flat, 32);
    s->ldfc = round_up(a.fc_units, 32);

    if (p.n_weights >= ((size_t)1 << 24) - 1) { err = "bf16 mode: more than 2^24 weights"; return SEED_ERR_UNSUPPORTED_ARCH; }
    Bf16Packed o;
    bf16_pack(p, s->torso_kind, s->ldf, s->ldfc, o);
    s->kc_fc = o.kc_fc; s->ft_fc = o.ft_fc; s->kc1_lstm = o.kc1_lstm; s->ft_hid = o.ft_hid;
    s->stack = o.stack;
    s->lw = o.lw;
    s->pk_bytes = o.pk.size() * 2;                // (one 16-bit element per table entry)
    s->fb_bytes = o.fb.size() * 4;
    const int F = a.fc_units;

    // arena layout
    auto al = [](size_t v) { return (v + 255) / 256 * 256; };
    const size_t mb = (size_t)a.max_batch;
    size_t off = 0;
    for (int set = 0; set < 2; ++set) {
        s->o_pk[set] = off; off += al(s->pk_bytes);
        s->o_fb[set] = off; off += al(s->fb_bytes + 16);
    }
    const size_t o_ko = off; off += al(o.ko.size() * 4 + 16);
    const size_t o_tpk = off; off += al(o.pk.size() * 4 + 16);
    const size_t o_tfb = off; off += al(o.fb.size() * 4 + 16);
    size_t o_act[2] = {0, 0};
    if (a.torso == SEED_TORSO_CONV_STACK && p.convs.size() > 1 && !s->stack_fused) {   // (the fused stack keeps them in LDS)
        size_t m = 0;
        for (size_t l = 0; l + 1 < p.convs.size(); ++l) {
            size_t n = (size_t)p.convs[l].OH * p.convs[l].OW * p.convs[l].Cout;
            if (n > m) m = n;
        }
        o_act[0] = off; off += al(mb * m * 2);
        o_act[1] = off; off += al(mb * m * 2);
    }
    size_t o_lw[4] = {0, 0, 0, 0};
    if (a.torso == SEED_TORSO_RESNET && s->torso_kind == TORSO_NONE) {
        size_t m0 = 0, m1 = 0;
        for (const Section& sec : p.sections) {
            m0 = std::max(m0, (size_t)sec.conv0.OH * sec.conv0.OW * sec.conv0.Cout);
            m1 = std::max(m1, (size_t)sec.PH * sec.PW * sec.conv0.Cout);
        }
        o_lw[0] = off; off += al(mb * m0 * 2);
        o_lw[1] = off; off += al(mb * m1 * 2);
        o_lw[2] = off; off += al(mb * m1 * 2);
        o_lw[3] = off; off += al(mb * m1 * 4);
    }
    const size_t o_feat = off; off += al(mb * s->ldf * 2);
    const size_t o_fcb = off; off += al(mb * s->ldfc * 2);
    const size_t o_fcf = off; off += al(mb * F * 4);
    BF_TRY(hipMalloc((void**)&s->arena, off));
    BF_TRY(hipMemset(s->arena, 0, off));      // padding columns of feat / fc stay zero for ever
    if (!o.pk.empty()) BF_TRY(hipMemcpy(s->arena + o_tpk, o.pk.data(), o.pk.size() * 4, hipMemcpyHostToDevice));
    if (!o.fb.empty()) BF_TRY(hipMemcpy(s->arena + o_tfb, o.fb.data(), o.fb.size() * 4, hipMemcpyHostToDevice));
    if (!o.ko.empty()) BF_TRY(hipMemcpy(s->arena + o_ko, o.ko.data(), o.ko.size() * 4, hipMemcpyHostToDevice));
    s->tab_pk = (const uint32_t*)(s->arena + o_tpk);
    s->tab_fb = (const uint32_t*)(s->arena + o_tfb);
    bf16_repack(s, d_w, 0, nullptr);
    BF_TRY(hipGetLastError());
    bf16_bind(s, p, o, 0);
    bf16_bind(s, p, o, 1);
    s->active = 0;
    s->koff = (const int*)(s->arena + o_ko);
    s->act[0] = (__bf16*)(s->arena + o_act[0]);
    s->act[1] = (__bf16*)(s->arena + o_act[1]);
    s->lw_c0 = (__bf16*)(s->arena + o_lw[0]);
    s->lw_r = (__bf16*)(s->arena + o_lw[1]);
    s->lw_u = (__bf16*)(s->arena + o_lw[2]);
    s->lw_x = (float*)(s->arena + o_lw[3]);
    s->feat = (__bf16*)(s->arena + o_feat);
    s->fc_bf16 = (__bf16*)(s->arena + o_fcb);
    s->fc_f32 = (float*)(s->arena + o_fcf);
    BF_TRY(gemm_lds_set_attributes<EPI_RELU>());
    BF_TRY(gemm_lds_set_attributes<EPI_LSTM>());

    // the LDS-tiled layer-by-layer convolution and the fused torso kernels may use more than 64 KiB of LDS
    BF_TRY(hipFuncSetAttribute((const void*)conv3x3_lds_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LT_LDS_MAX));
    BF_TRY(hipFuncSetAttribute((const void*)conv3x3_lds_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LT_LDS_MAX));
    BF_TRY(hipFuncSetAttribute((const void*)conv3x3_lds_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LT_LDS_MAX));
    {
        // the per-section kernels of the layer-by-layer ResNet path may ask for more than 64 KiB as well
        hipError_t e = hipSuccess;
        auto set = [&](const void* f, size_t bytes) {
            if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        };
        set((const void*)conv_pool_kernel<16, 16>, CP_LDS_MAX);
        set((const void*)conv_pool_kernel<16, 32>, CP_LDS_MAX);
        set((const void*)conv_pool_kernel<32, 32>, CP_LDS_MAX);
        set((const void*)conv_pool_kernel<32, 64>, CP_LDS_MAX);
        set((const void*)conv_pool_kernel<64, 64>, CP_LDS_MAX);
        set((const void*)conv_pool_kernel<64, 128>, CP_LDS_MAX);
        set((const void*)conv_pool_kernel<128, 128>, CP_LDS_MAX);
        set((const void*)conv_tile_kernel<128, true>, CT_LDS_MAX);
        set((const void*)conv_tile_kernel<128, false>, CT_LDS_MAX);
        set((const void*)first_pool_kernel<64, 4>, FirstPoolCfg<64, 4>::LDS_MAX);
        set((const void*)first_pool_kernel<64, 8>, FirstPoolCfg<64, 8>::LDS_MAX);
        set((const void*)first_pool_kernel<64, 16>, FirstPoolCfg<64, 16>::LDS_MAX);
        BF_TRY(e);
    }
    BF_TRY(hipFuncSetAttribute((const void*)resblock_fused_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)RB_LDS_MAX));
    BF_TRY(hipFuncSetAttribute((const void*)resblock_fused_kernel<32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)RB_LDS_MAX));
    BF_TRY(hipFuncSetAttribute((const void*)resblock_fused_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)RB_LDS_MAX));
    BF_TRY(hipFuncSetAttribute((const void*)resblock_fused_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)RB_LDS_MAX));
    if (s->stack_fused) {
        BF_TRY(hipFuncSetAttribute((const void*)r2d2_torso_bf16_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, r2d2::LDS_BYTES));
        BF_TRY(hipFuncSetAttribute((const void*)r2d2_torso_bf16_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, r2d2::LDS_BYTES));
    }
    if (s->torso_kind == TORSO_DMLAB) {
        BF_TRY(hipFuncSetAttribute((const void*)resnet3_bf16_kernel<DmS1, DmS2, DmS3>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, Net3<DmS1, DmS2, DmS3>::LDS_BYTES));
    } else if (s->torso_kind == TORSO_FOOTBALL) {
        BF_TRY(hipFuncSetAttribute((const void*)resnet4_bf16_kernel<FbS1, DmS2, DmS3, FbS4>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, Net4<FbS1, DmS2, DmS3, FbS4>::LDS_BYTES));
    }
    return SEED_OK;
}

// Large batch: LDS-staged tiles.
template <int EPI>
inline bool launch_gemm_lds(hipStream_t st, const GemmArgs& g, int tile_groups, int n_cu)
{
    if (g.rows < GL_MIN_ROWS || (g.kc1 & 1)) return false;
    const int kct = g.kc1 + (g.k2 + 31) / 32;
    if constexpr (EPI == EPI_RELU) {
        // 64 x 64 tiles with K over the eight wavefronts where wider tiles would be too few for the chip: long K
        // (the linear layer after the torso) with fewer 128 x 256 tiles than compute units, and shorter K with
        // fewer 64 x 256 tiles than half the units (the Football agent's 960 -> 256 layer at 2048 rows: 6.9 us
        // against 16.2 with 32 tiles of 64 x 256)
        const long wide = (long)((g.rows + 127) / 128) * ((tile_groups + 3) / 4);
        const long mid = (long)((g.rows + 63) / 64) * ((tile_groups + 3) / 4);
        if (g.k2 == 0 && ((kct >= 64 && wide < n_cu) || (kct >= 16 && kct < 64 && mid < n_cu / 2))) {
            hipLaunchKernelGGL((gemm_bf16_k8_kernel<EPI>), dim3((g.rows + 63) / 64, tile_groups), dim3(GL_THREADS), GL_K8_LDS_BYTES, st, g);
            return true;
        }
    }
    const int by = (tile_groups + 3) / 4;
    constexpr int LDS42 = GemmXwCfg<4, 2, 1, true>::LDS_BYTES, LDS41 = GemmXwCfg<4, 1, 2, true>::LDS_BYTES;
    if ((long)((g.rows + 127) / 128) * by >= n_cu)
        hipLaunchKernelGGL((gemm_bf16_xw_kernel<4, 2, 1, EPI, true>), dim3((g.rows + 127) / 128, by), dim3(GL_THREADS), LDS42, st, g);
    else
        hipLaunchKernelGGL((gemm_bf16_xw_kernel<4, 1, 2, EPI, true>), dim3((g.rows + 63) / 64, by), dim3(GL_THREADS), LDS41, st, g);
    return true;
}

template <int EPI>
inline void launch_gemm(hipStream_t st, const GemmArgs& g, int tile_groups, int n_cu)
{
    if (launch_gemm_lds<EPI>(st, g, tile_groups, n_cu)) return;
    // RT (row tiles of 16 per wavefront / block): the largest that still gives every compute unit two blocks
    const long want = 2L * n_cu;
    const int kct = g.kc1 + (g.k2 + 31) / 32;
    // (the LSTM of a 512-unit core has 32 chunks: for it the kernels below were measured faster from 512 rows on -
    // 13.9 vs 16.2 us at 512 rows, 35 vs 60 us at 1984 - and equal below, so its gates take the long-K path from 64 chunks)
    if (kct >= (EPI == EPI_LSTM ? 64 : 32)) {
        // long K: one block per (RT*16 rows, 4 feature tiles), K split over its wavefronts.  The loop is bound by
        // the load instructions each compute unit issues, so the largest tile that still gives every compute
        // unit a block wins, with 8 wavefronts to keep enough loads in flight.
        const int gy = tile_groups;
        auto go = [&](auto rt, auto nw) {
            constexpr int RT = decltype(rt)::value, NW = decltype(nw)::value;
            hipLaunchKernelGGL((gemm_bf16_splitk_kernel<RT, EPI, NW>), dim3((g.rows + RT * 16 - 1) / (RT * 16), gy), dim3(NW * 64),
                               4 * RT * 4 * 64 * sizeof(floatx4), st, g);
        };
        using W4 = std::integral_constant<int, 4>; using W8 = std::integral_constant<int, 8>;
        if constexpr (EPI == EPI_RELU) {
            // small batches: the finest output tiles (16 x 16, else 16 x 32) that still number no more than the
            // compute units: the kernel's time is the weight bytes one unit pulls (measured, K = 3456: 5.8 / 6.9 /
            // 8.9 us for 16 / 32 / 64 features per tile, whatever the rows, until the tiles outnumber the units -
            // then it doubles)
            const long rt16 = (g.rows + 15) / 16;
            if (rt16 * g.n_ftiles <= n_cu) {
                hipLaunchKernelGGL((gemm_bf16_splitk_kernel<1, EPI, 4, 1>), dim3(rt16, g.n_ftiles), dim3(256),
                                   4 * 1 * 4 * 64 * sizeof(floatx4), st, g);
                return;
            }
            if (rt16 * ((g.n_ftiles + 1) / 2) <= n_cu) {
                hipLaunchKernelGGL((gemm_bf16_splitk_kernel<1, EPI, 4, 2>), dim3(rt16, (g.n_ftiles + 1) / 2), dim3(256),
                                   4 * 1 * 4 * 64 * sizeof(floatx4), st, g);
                return;
            }
        }
        if ((long)((g.rows + 63) / 64) * gy >= n_cu) go(std::integral_constant<int, 4>{}, W8{});
        else if ((long)((g.rows + 31) / 32) * gy >= n_cu) go(std::integral_constant<int, 2>{}, W8{});
        else go(std::integral_constant<int, 1>{}, W4{});
    } else {
        // small batches: one tile group per block with K split over its four wavefronts puts four times as many
        // compute units to work as the group-per-wavefront kernel below (measured: 4.9 vs 8.1 us at 64 rows, 6.2 vs
        // 8.2 at 512, slower at 1024)
        if ((long)((g.rows + 15) / 16) * tile_groups <= want) {
            hipLaunchKernelGGL((gemm_bf16_splitk_kernel<1, EPI, 4>), dim3((g.rows + 15) / 16, tile_groups), dim3(256),
                               4 * 1 * 4 * 64 * sizeof(floatx4), st, g);
            return;
        }
        // otherwise a tile group per wavefront, whole K: the largest row tile that still gives (nearly) every compute
        // unit a block (measured, 512-unit LSTM at 1984 rows: 35 / 36 / 43 us with 248 / 496 / 992 blocks)
        const int gy = (tile_groups + 3) / 4;
        const long enough = (long)n_cu * 7 / 8;
        if ((long)((g.rows + 63) / 64) * gy >= enough) hipLaunchKernelGGL((gemm_bf16_kernel<4, EPI>), dim3((g.rows + 63) / 64, gy), dim3(256), 0, st, g);
        else if ((long)((g.rows + 31) / 32) * gy >= enough) hipLaunchKernelGGL((gemm_bf16_kernel<2, EPI>), dim3((g.rows + 31) / 32, gy), dim3(256), 0, st, g);
        else hipLaunchKernelGGL((gemm_bf16_kernel<1, EPI>), dim3((g.rows + 15) / 16, gy), dim3(256), 0, st, g);
    }
}

template <int FT, bool U8>
inline void launch_conv_stack(hipStream_t st, const ConvStackArgs& c)
{
    const long npix = (long)c.B * c.OH * c.OW;
    const int gy = c.Cout / (16 * FT);
    if (npix >= 65536) hipLaunchKernelGGL((conv_stack_bf16_kernel<FT, 2, U8>), dim3((unsigned)((npix + 127) / 128), gy), dim3(256), 0, st, c);
    else hipLaunchKernelGGL((conv_stack_bf16_kernel<FT, 1, U8>), dim3((unsigned)((npix + 63) / 64), gy), dim3(256), 0, st, c);
}

inline void launch_lw_conv(hipStream_t st, const LwConvArgs& c, int ft, bool u8)
{
    const long npix = (long)c.B * c.H * c.W;
    const int gy = c.Cout / (16 * ft);
    if (!u8 && c.Cin % 32 == 0 && lt_lds_bytes(c.W, c.Cin) <= LT_LDS_MAX) {
        // bf16 input with whole 32-channel chunks: the LDS-tiled kernel
        const int hw = c.H * c.W;
        const dim3 grid((unsigned)(c.B * ((hw + LT_PIX - 1) / LT_PIX)), gy);
        const size_t lds = lt_lds_bytes(c.W, c.Cin);
        const int plane = lt_plane_cells(c.W);
        if (ft == 4) hipLaunchKernelGGL(conv3x3_lds_kernel<4>, grid, dim3(LT_THREADS), lds, st, c, plane);
        else if (ft == 2) hipLaunchKernelGGL(conv3x3_lds_kernel<2>, grid, dim3(LT_THREADS), lds, st, c, plane);
        else hipLaunchKernelGGL(conv3x3_lds_kernel<1>, grid, dim3(LT_THREADS), lds, st, c, plane);
        return;
    }
    auto go = [&](auto ftc, auto rtc, auto u8c) {
        constexpr int FT = decltype(ftc)::value, RT = decltype(rtc)::value;
        constexpr bool U8 = decltype(u8c)::value;
        hipLaunchKernelGGL((conv3x3_lw_kernel<FT, RT, U8>), dim3((unsigned)((npix + 64 * RT - 1) / (64 * RT)), gy), dim3(256), 0, st, c);
    };
    auto by_rt = [&](auto ftc, auto u8c) {
        if (npix >= 65536) go(ftc, std::integral_constant<int, 2>{}, u8c);
        else go(ftc, std::integral_constant<int, 1>{}, u8c);
    };
    auto by_ft = [&](auto u8c) {
        if (ft == 4) by_rt(std::integral_constant<int, 4>{}, u8c);
        else if (ft == 2) by_rt(std::integral_constant<int, 2>{}, u8c);
        else by_rt(std::integral_constant<int, 1>{}, u8c);
    };
    if (u8) by_ft(std::true_type{});
    else by_ft(std::false_type{});
}

// The first layer with its pooling as one launch (uint8 frame -> fp32 x and, if r is given, ReLU(x) as bf16);
// false when the layer has no fused kernel, and nothing was launched.
inline bool launch_first_pool(hipStream_t st, const LwLayerDev& d, const bf16x8* wp_conv, const float* d_w, const Section& sec, int B,
                              const uint8_t* obs, float* x, __bf16* r)
{
    const ConvLayer& c = sec.conv0;
    if (d.first_off == LW_NONE) return false;
    auto go = [&](auto cc, auto cellc) -> bool {
        constexpr int CC = decltype(cc)::value, CELL = decltype(cellc)::value;
        using K = FirstPoolCfg<CC, CELL>;
        FirstPoolArgs a{};
        if (!K::choose(sec.PH, sec.PW, a.PTH, a.PTW)) return false;
        if (CELL != 4 && d.kchunks != K::KCH) return false;
        a.obs = obs; a.wp = wp_conv + d.first_off / 8; a.bias = d_w + c.b_off; a.scale = 1.0f / 255.0f;
        a.x = x; a.r = r;
        a.B = B; a.H = c.H; a.W = c.W; a.Cin = c.Cin; a.PH = sec.PH; a.PW = sec.PW; a.pad_h = sec.pool_pad_h; a.pad_w = sec.pool_pad_w;
        a.tiles_y = (sec.PH + a.PTH - 1) / a.PTH; a.tiles_x = (sec.PW + a.PTW - 1) / a.PTW;
        hipLaunchKernelGGL((first_pool_kernel<CC, CELL>), dim3((unsigned)((long)B * a.tiles_y * a.tiles_x)), dim3(FP_THREADS),
                           K::lds_bytes(a.PTH, a.PTW), st, a);
        return true;
    };
    auto by_cell = [&](auto cc) -> bool {
        if (c.Cin <= 4) return go(cc, std::integral_constant<int, 4>{});
        if (c.Cin == 8) return go(cc, std::integral_constant<int, 8>{});
        if (c.Cin == 16) return go(cc, std::integral_constant<int, 16>{});
        return false;
    };
    switch (c.Cout) {
    case 16: return by_cell(std::integral_constant<int, 16>{});
    case 32: return by_cell(std::integral_constant<int, 32>{});
    case 64: return by_cell(std::integral_constant<int, 64>{});
    default: return false;
    }
}

// conv0 of a later section with its pooling as one launch (bf16 NHWC map -> fp32 x and, if r is given, ReLU(x) as
// bf16); false when the channel pair has no fused kernel or no tile fits, and nothing was launched.
template <class F>
inline bool conv_pool_by_channels(int cin, int cout, F go)
{
    auto pair = [&](auto ci, auto co) { return go(ci, co); };
    using I16 = std::integral_constant<int, 16>; using I32 = std::integral_constant<int, 32>;
    using I64 = std::integral_constant<int, 64>; using I128 = std::integral_constant<int, 128>;
    switch (cin * 1000 + cout) {
    case 16016: return pair(I16{}, I16{});
    case 16032: return pair(I16{}, I32{});
    case 32032: return pair(I32{}, I32{});
    case 32064: return pair(I32{}, I64{});
    case 64064: return pair(I64{}, I64{});
    case 64128: return pair(I64{}, I128{});
    case 128128: return pair(I128{}, I128{});
    default: return false;
    }
}

inline bool launch_conv_pool(hipStream_t st, const LwLayerDev& d, const bf16x8* wp_conv, const float* d_w, const Section& sec, int B,
                             const __bf16* in, float* x, __bf16* r)
{
    const ConvLayer& c = sec.conv0;
    return conv_pool_by_channels(c.Cin, c.Cout, [&](auto ci, auto co) -> bool {
        constexpr int CIN = decltype(ci)::value, COUT = decltype(co)::value;
        using CP = ConvPoolCfg<CIN, COUT>;
        ConvPoolArgs a{};
        if (!CP::choose(sec.PH, sec.PW, a.PTH, a.PTW)) return false;
        a.in = in; a.wp = wp_conv + d.wp_off / 8; a.bias = d_w + c.b_off; a.x = x; a.r = r;
        a.B = B; a.H = c.H; a.W = c.W; a.PH = sec.PH; a.PW = sec.PW; a.pad_h = sec.pool_pad_h; a.pad_w = sec.pool_pad_w;
        a.tiles_y = (sec.PH + a.PTH - 1) / a.PTH; a.tiles_x = (sec.PW + a.PTW - 1) / a.PTW; a.kchunks = d.kchunks;
        hipLaunchKernelGGL((conv_pool_kernel<CIN, COUT>), dim3((unsigned)((long)B * a.tiles_y * a.tiles_x)), dim3(RB_THREADS),
                           CP::lds_bytes(a.PTH, a.PTW), st, a);
        return true;
    });
}

template <class F>
inline bool resblock_by_width(int C, F go)
{
    switch (C) {
    case 16: return go(std::integral_constant<int, 16>{});
    case 32: return go(std::integral_constant<int, 32>{});
    case 64: return go(std::integral_constant<int, 64>{});
    case 128: return go(std::integral_constant<int, 128>{});
    default: return false;
    }
}

// Blocks that run as two conv_tile_kernel launches.  Measured at 1024 images against the one-launch block: 128
// channels (18 x 24 and 9 x 12, mean) 108 + 137 us vs 306; 64 channels on 36 x 48 219 + 323 vs 505, on 18 x 24 and
// 9 x 12 42 + 52 vs 84 - so 128 channels only.
inline bool conv_tile_preferred(const ConvLayer& c) { return c.Cin == c.Cout && c.Cin == 128; }

// pitch-wide regions (conflict-free map fragments) where measured faster: 64 channels on maps larger than 18 x 24
inline bool resblock_flat(const ConvLayer& c) { return c.Cin == 64 && c.H * c.W > 18 * 24; }

// Whether launch_resblock takes this block: every width with a kernel whose tile fits.  Measured at 1024 images
// against the two-launch form (LDS-tiled convolution kernel twice): 16 ch 54 x 72 149 vs 308 us; 32 ch 36 x 48 175
// vs 284, 27 x 36 and smaller 52 vs 70; 64 ch 36 x 48 552 vs 640, 18 x 24 and 9 x 12 84 vs 124; 128 ch (18 x 24 and
// 9 x 12, mean) 305 vs 412.
inline bool resblock_fusable(const ConvLayer& ca, const ConvLayer& cb)
{
    const int C = ca.Cin;
    if (ca.Cout != C || cb.Cin != C || cb.Cout != C || ca.H != cb.H || ca.W != cb.W) return false;
    return resblock_by_width(C, [&](auto cc) {
        int th, tw;
        return ResBlockCfg<decltype(cc)::value>::choose(ca.H, ca.W, resblock_flat(ca), th, tw);
    });
}

// One residual block (two 3x3 convolutions C -> C over an H x W map) as a single launch; false when the width has
// no fused kernel or no tile fits, and nothing was launched.
inline bool launch_resblock(hipStream_t st, const LwLayerDev& da, const LwLayerDev& db, const bf16x8* wp_conv, const float* d_w,
                            const ConvLayer& ca, const ConvLayer& cb, int B, const float* x_in, float* x_out, __bf16* y, int y_relu,
                            int ldy)
{
    if (!resblock_fusable(ca, cb)) return false;
    return resblock_by_width(ca.Cin, [&](auto cc) -> bool {
        constexpr int CC = decltype(cc)::value;
        using K = ResBlockCfg<CC>;
        ResBlockArgs r{};
        r.flat = resblock_flat(ca);
        if (!K::choose(ca.H, ca.W, r.flat != 0, r.TH, r.TW)) return false;
        r.x_in = x_in; r.wpa = wp_conv + da.wp_off / 8; r.wpb = wp_conv + db.wp_off / 8;
        r.bias_a = d_w + ca.b_off; r.bias_b = d_w + cb.b_off;
        r.x_out = x_out; r.y = y; r.y_relu = y_relu; r.ldy = ldy;
        r.B = B; r.H = ca.H; r.W = ca.W; r.kchunks = da.kchunks;
        r.tiles_y = (ca.H + r.TH - 1) / r.TH; r.tiles_x = (ca.W + r.TW - 1) / r.TW;
        hipLaunchKernelGGL(resblock_fused_kernel<CC>, dim3((unsigned)((long)B * r.tiles_y * r.tiles_x)), dim3(RB_THREADS),
                           K::lds_bytes(r.TH, r.TW, r.flat != 0), st, r);
        return true;
    });
}

// One convolution of a residual block as a launch of its own over large LDS tiles (conv_tile_kernel); false when
// the width has no such kernel or no tile fits, and nothing was launched.
inline bool launch_conv_tile(hipStream_t st, const LwLayerDev& d, const bf16x8* wp_conv, const float* d_w, const ConvLayer& c, int B,
                             const void* in, bool in_f32, const float* resid, float* x_out, __bf16* y, int y_relu, int ldy)
{
    if (c.Cin != c.Cout) return false;
    auto go = [&](auto cc) -> bool {
        constexpr int CC = decltype(cc)::value;
        using CT = ConvTileCfg<CC>;
        ConvTileArgs a{};
        if (d.kchunks != (9 * CC + 31) / 32 || !CT::choose(c.H, c.W, a.TH, a.TW)) return false;
        a.in = in; a.wp = wp_conv + d.wp_off / 8; a.bias = d_w + c.b_off; a.resid = resid; a.x_out = x_out; a.y = y;
        a.y_relu = y_relu; a.ldy = ldy;
        a.B = B; a.H = c.H; a.W = c.W; a.kchunks = d.kchunks;
        a.tiles_y = (c.H + a.TH - 1) / a.TH; a.tiles_x = (c.W + a.TW - 1) / a.TW;
        const dim3 grid((unsigned)((long)B * a.tiles_y * a.tiles_x));
        if (in_f32) hipLaunchKernelGGL((conv_tile_kernel<CC, true>), grid, dim3(RB_THREADS), CT::lds_bytes(a.TH, a.TW), st, a);
        else hipLaunchKernelGGL((conv_tile_kernel<CC, false>), grid, dim3(RB_THREADS), CT::lds_bytes(a.TH, a.TW), st, a);
        return true;
    };
    switch (c.Cin) {
    case 128: return go(std::integral_constant<int, 128>{});
    default: return false;
    }
}

// Torso and linear layer over B rows: leaves the rectified linear-layer output of row r in row r of
// fc_bf16 / fc_f32.
inline seed_status_t bf16_torso_fc(Bf16State* s, const Plan& p, const float* d_w, hipStream_t st, int B, const uint8_t* obs,
                                   hipEvent_t ev0, hipEvent_t ev1, std::string& err)
{
    const seed_arch_t& a = p.arch;
    const Bf16WeightSet& W = s->ws[s->active];
    if (ev0) (void)hipEventRecord(ev0, st);
    if (a.torso == SEED_TORSO_RESNET && s->torso_kind == TORSO_NONE) {
        // layer by layer: conv0 -> pool -> (conv_a, conv_b) x 2 per section, activations in HBM
        const void* in = obs;
        size_t li = 0;
        for (size_t si = 0; si < p.sections.size(); ++si) {
            const Section& sec = p.sections[si];
            const bool last_sec = si + 1 == p.sections.size();
            auto conv = [&](const ConvLayer& c, const void* src, bool u8, const float* x_in, float* x_out, __bf16* y, int y_relu,
                            int ldy) {
                const LwLayerDev& d = s->lw[li++];
                LwConvArgs ca{};
                ca.in = src; ca.wp = W.wp_conv + d.wp_off / 8; ca.bias = d_w + c.b_off;
                ca.ktab = (const int2*)(s->koff + d.ktab_off);
                ca.x_in = x_in; ca.x_out = x_out; ca.y = y; ca.y_relu = y_relu; ca.ldy = ldy;
                ca.B = B; ca.H = c.H; ca.W = c.W; ca.Cin = c.Cin; ca.Cout = c.Cout; ca.kchunks = d.kchunks;
                ca.scale = u8 ? 1.0f / 255.0f : 1.0f;
                const int nft = c.Cout / 16;
                const int ft = nft % 4 == 0 ? 4 : (nft % 2 == 0 ? 2 : 1);
                launch_lw_conv(st, ca, ft, u8);
            };
            // only the layer-by-layer block convolutions read R; a fused block takes ReLU(x) itself
            const bool need_r = !resblock_fusable(sec.block[0], sec.block[1]);
            if (si == 0 && launch_first_pool(st, s->lw[li], W.wp_conv, d_w, sec, B, obs, s->lw_x, need_r ? s->lw_r : nullptr)) {
                ++li;
            } else if (si > 0 && !need_r && launch_conv_pool(st, s->lw[li], W.wp_conv, d_w, sec, B, (const __bf16*)in, s->lw_x, nullptr)) {
                // (not when R is wanted: it would land in lw_r, which is this layer's input)
                ++li;
            } else {
                conv(sec.conv0, in, si == 0, nullptr, nullptr, s->lw_c0, 0, 0);
                const int C = sec.conv0.Cout;
                const long total = (long)B * sec.PH * sec.PW * (C / 4);
                hipLaunchKernelGGL(pool3x3s2_lw_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s->lw_c0, s->lw_x,
                                   need_r ? s->lw_r : nullptr, B, sec.conv0.OH, sec.conv0.OW, C, sec.PH, sec.PW, sec.pool_pad_h, sec.pool_pad_w);
            }
            // a residual block in one launch where the width has a fused kernel and a tile fits; x ping-pongs between
            // lw_x and the (by now dead) conv0 map, since tiles read their neighbours' halos of the block's input
            float* x_cur = s->lw_x;
            float* x_alt = (float*)s->lw_c0;
            for (int blk = 0; blk < 2; ++blk) {
                const bool closing = last_sec && blk == 1;          // the torso's last layer writes the rectified features
                const bool to_next = !last_sec && blk == 1;         // the next section's conv0 takes x un-rectified
                __bf16* y = closing ? s->feat : s->lw_r;
                const int y_relu = to_next ? 0 : 1, ldy = closing ? s->ldf : 0;
                // (two launches over larger tiles where the one-launch block is bound by operand delivery; conv_b adds
                // and writes x in place: it reads no pixel of x but its own)
                if (conv_tile_preferred(sec.block[2 * blk]) &&
                    launch_conv_tile(st, s->lw[li], W.wp_conv, d_w, sec.block[2 * blk], B, x_cur, true, nullptr, nullptr, s->lw_u, 1, 0)) {
                    if (!launch_conv_tile(st, s->lw[li + 1], W.wp_conv, d_w, sec.block[2 * blk + 1], B, s->lw_u, false, x_cur,
                                          blk == 0 ? x_cur : nullptr, blk == 0 ? nullptr : y, y_relu, ldy)) {
                        err = "residual block: second convolution has no tile kernel";
                        return SEED_ERR_DEVICE;
                    }
                    li += 2;
                    continue;
                }
                if (launch_resblock(st, s->lw[li], s->lw[li + 1], W.wp_conv, d_w, sec.block[2 * blk], sec.block[2 * blk + 1], B, x_cur,
                                    blk == 0 ? x_alt : nullptr, blk == 0 ? nullptr : y, y_relu, ldy)) {
                    li += 2;
                    if (blk == 0) std::swap(x_cur, x_alt);
                    continue;
                }
                if (x_cur != s->lw_x) {                             // unreachable: both blocks of a section have one shape
                    err = "residual blocks of one section differ in shape";
                    return SEED_ERR_DEVICE;
                }
                conv(sec.block[2 * blk], s->lw_r, false, nullptr, nullptr, s->lw_u, 1, 0);
                conv(sec.block[2 * blk + 1], s->lw_u, false, s->lw_x, s->lw_x, y, y_relu, ldy);
            }
            in = s->lw_r;
        }
    } else if (a.torso == SEED_TORSO_RESNET) {
        TorsoArgs t{};
        t.obs = obs; t.feat = s->feat; t.ldf = s->ldf; t.B = B;
        for (int i = 0; i < 4; ++i) t.sec[i] = W.sec[i];
        const int grid = B < s->n_cu ? B : s->n_cu;
        constexpr int LDS_DM = Net3<DmS1, DmS2, DmS3>::LDS_BYTES;
        constexpr int LDS_FB = Net4<FbS1, DmS2, DmS3, FbS4>::LDS_BYTES;
        static_assert(LDS_DM <= 160 * 1024 && LDS_FB <= 160 * 1024, "torso does not fit the 160 KiB of LDS");
        if (s->torso_kind == TORSO_DMLAB)
            hipLaunchKernelGGL((resnet3_bf16_kernel<DmS1, DmS2, DmS3>), dim3(grid), dim3(RN_THREADS), LDS_DM, st, t);
        else
            hipLaunchKernelGGL((resnet4_bf16_kernel<FbS1, DmS2, DmS3, FbS4>), dim3(grid), dim3(RN_THREADS), LDS_FB, st, t);
    } else if (s->stack_fused) {
        R2d2TorsoArgs t{};
        t.obs = obs; t.feat = s->feat; t.ldf = s->ldf; t.B = B;
        t.w1 = W.wp_conv + s->stack[0].wp_off / 8; t.w2 = W.wp_conv + s->stack[1].wp_off / 8; t.w3 = W.wp_conv + s->stack[2].wp_off / 8;
        t.b1 = d_w + p.convs[0].b_off; t.b2 = d_w + p.convs[1].b_off; t.b3 = d_w + p.convs[2].b_off;
        const dim3 grid(B < s->n_cu ? B : s->n_cu);
        if (a.obs_c == 4) hipLaunchKernelGGL(r2d2_torso_bf16_kernel<4>, grid, dim3(r2d2::THREADS), r2d2::LDS_BYTES, st, t);
        else hipLaunchKernelGGL(r2d2_torso_bf16_kernel<1>, grid, dim3(r2d2::THREADS), r2d2::LDS_BYTES, st, t);
    } else {
        const void* x = obs;
        for (size_t l = 0; l < p.convs.size(); ++l) {
            const ConvLayer& c = p.convs[l];
            const bool last = l + 1 == p.convs.size();
            ConvStackArgs ca{};
            ca.x = x; ca.wp = W.wp_conv + s->stack[l].wp_off / 8; ca.bias = d_w + c.b_off;
            ca.koff = s->koff + s->stack[l].koff_off; ca.y = last ? s->feat : s->act[l & 1];
            ca.B = B; ca.H = c.H; ca.W = c.W; ca.Cin = c.Cin; ca.OH = c.OH; ca.OW = c.OW; ca.Cout = c.Cout;
            ca.stride = c.stride; ca.kchunks = s->stack[l].kchunks; ca.scale = l == 0 ? 1.0f / 255.0f : 1.0f;
            const int nft = c.Cout / 16;
            const int ft = nft % 4 == 0 ? 4 : (nft % 2 == 0 ? 2 : 1);
            if (l == 0) {
                if (ft == 4) launch_conv_stack<4, true>(st, ca); else if (ft == 2) launch_conv_stack<2, true>(st, ca); else launch_conv_stack<1, true>(st, ca);
            } else {
                if (ft == 4) launch_conv_stack<4, false>(st, ca); else if (ft == 2) launch_conv_stack<2, false>(st, ca); else launch_conv_stack<1, false>(st, ca);
            }
            x = ca.y;
        }
    }
    if (ev1) (void)hipEventRecord(ev1, st);
    // linear layer + ReLU -> bf16 (for the core GEMM) and fp32 (for heads / taps)
    {
        GemmArgs g{};
        g.x1 = s->feat; g.ld1 = s->ldf; g.kc1 = s->kc_fc; g.k2 = 0;
        g.wp = W.wp_fc; g.n_ftiles = s->ft_fc; g.rows = B; g.bias_pad = W.bias_fc;
        g.y_bf16 = s->fc_bf16; g.ldy_bf16 = s->ldfc; g.y_f32 = s->fc_f32; g.ldy_f32 = a.fc_units; g.n_out = a.fc_units;
        launch_gemm<EPI_RELU>(st, g, (s->ft_fc + 3) / 4, s->n_cu);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { err = std::string("kernel launch: ") + hipGetErrorString(e); return SEED_ERR_DEVICE; }
    return SEED_OK;
}

// Recurrent core and dueling hidden layers for the B rows that start at row `row0` of the linear layer's
// output (the caller's pointers already name those rows' own inputs and outputs).  On return *core /
// *ld_core name the fp32 rows the output heads read.
inline seed_status_t bf16_core(Bf16State* s, const Plan& p, const float* d_w, hipStream_t st, int row0, int B,
                               const int32_t* prev_action, const float* prev_reward, const float* h_in,
                               const float* c_in, const uint8_t* done, float* h_out, float* c_out, float* d_hid,
                               const float** core, int* ld_core, std::string& err, bool do_core = true, bool do_hidden = true)
{
    const seed_arch_t& a = p.arch;
    const Bf16WeightSet& W = s->ws[s->active];
    const __bf16* fc_bf16 = s->fc_bf16 + (size_t)row0 * s->ldfc;
    *core = s->fc_f32 + (size_t)row0 * a.fc_units; *ld_core = a.fc_units;
    if (a.lstm_units > 0 && !do_core) { *core = h_out; *ld_core = a.lstm_units; }
    if (a.lstm_units > 0 && do_core) {
        GemmArgs g{};
        g.x1 = fc_bf16; g.ld1 = s->ldfc; g.kc1 = s->kc1_lstm;
        g.x2 = h_in; g.ld2 = a.lstm_units; g.k2 = a.lstm_units;
        g.wp = W.wp_lstm; g.n_ftiles = (a.lstm_units / 16) * 4; g.rows = B;
        g.lstm_w = d_w + p.lstm_w; g.lstm_b = d_w + p.lstm_b; g.prev_action = prev_action; g.prev_reward = prev_reward;
        g.c_in = c_in; g.h_out = h_out; g.c_out = c_out; g.F = a.fc_units; g.A = a.num_actions; g.Hn = a.lstm_units;
        g.done = done;
        launch_gemm<EPI_LSTM>(st, g, a.lstm_units / 16, s->n_cu);
        *core = h_out; *ld_core = a.lstm_units;
    }
    if (a.head == SEED_HEAD_DUELING_Q && do_hidden) {
        GemmArgs g{};
        if (a.lstm_units > 0) { g.kc1 = 0; g.x1 = fc_bf16; g.ld1 = s->ldfc; g.x2 = h_out; g.ld2 = a.lstm_units; g.k2 = a.lstm_units; }
        else { g.x1 = fc_bf16; g.ld1 = s->ldfc; g.kc1 = s->ldfc / 32; g.k2 = 0; }
        g.wp = W.wp_hid; g.n_ftiles = s->ft_hid; g.rows = B; g.bias_pad = W.bias_hid;
        g.y_bf16 = nullptr; g.y_f32 = d_hid; g.ldy_f32 = 2 * a.head_hidden; g.n_out = 2 * a.head_hidden;
        launch_gemm<EPI_RELU>(st, g, (s->ft_hid + 3) / 4, s->n_cu);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { err = std::string("kernel launch: ") + hipGetErrorString(e); return SEED_ERR_DEVICE; }
    return SEED_OK;
}

// One step: torso, linear layer, recurrent core and dueling hidden layers.
inline seed_status_t bf16_step(Bf16State* s, const Plan& p, const float* d_w, hipStream_t st, int B, const uint8_t* obs,
                               const int32_t* prev_action, const float* prev_reward, const float* h_in,
                               const float* c_in, const uint8_t* done, float* h_out, float* c_out, float* d_hid,
                               const float** core, int* ld_core, hipEvent_t ev0, hipEvent_t ev1, std::string& err)
{
    const seed_status_t st0 = bf16_torso_fc(s, p, d_w, st, B, obs, ev0, ev1, err);
    if (st0 != SEED_OK) return st0;
    return bf16_core(s, p, d_w, st, 0, B, prev_action, prev_reward, h_in, c_in, done, h_out, c_out, d_hid, core, ld_core, err);
}

inline seed_status_t bf16_read_intermediate(Bf16State* s, const Plan& p, int which, int B, float* dst, hipStream_t st,
                                            std::string& err)
{
    (void)err;
    if (which == 0) {
        size_t total = (size_t)B * p.flat;
        hipLaunchKernelGGL(bf16_rows_to_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s->feat, s->ldf, dst,
                           (int)p.flat, total);
    } else {
        size_t total = (size_t)B * p.arch.fc_units;
        hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s->fc_f32, dst, total);
    }
    return SEED_OK;
}

}  // namespace seedinf
