// Host-side network plan: turns a seed_arch_t into an ordered list of layers
// with shapes and offsets into the canonical flat weight vector.  No device
// code here.
#pragma once
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/seedinf.h"

namespace seedinf {

struct ConvLayer {
    int H, W, Cin;        // input extent
    int OH, OW, Cout;     // output extent
    int k, stride, pad;   // pad = leading zero padding (0 for "valid", 1 for 3x3 SAME)
    size_t w_off, b_off;  // offsets (floats) into the flat weights
};

struct Section {          // one deep-ResNet section
    ConvLayer conv0;      // 3x3 SAME, Cin -> C
    int PH, PW;           // extent after the 3x3 / stride-2 SAME max-pool
    int pool_pad_h, pool_pad_w;   // leading pool padding (0 or 1)
    ConvLayer block[4];   // block1.a, block1.b, block2.a, block2.b (3x3 SAME, C -> C at PH x PW)
};

struct Plan {
    seed_arch_t arch{};
    std::vector<ConvLayer> convs;      // conv-stack torso
    std::vector<Section> sections;     // ResNet torso
    int feat_h = 0, feat_w = 0, feat_c = 0;
    size_t flat = 0;                   // torso features per row
    size_t fc_w = 0, fc_b = 0;
    // LSTM: rows [fc features | action rows | reward row | h rows], 4H columns
    size_t lstm_w = 0, lstm_b = 0;
    int core = 0;                      // width of the core output fed to the heads
    // heads
    size_t pol_w = 0, pol_b = 0, val_w = 0, val_b = 0;                // policy / value
    size_t v1_w = 0, v1_b = 0, v2_w = 0, v2_b = 0;                    // dueling value stream
    size_t a1_w = 0, a1_b = 0, a2_w = 0, a2_b = 0;                    // dueling advantage stream
    size_t n_weights = 0;
    size_t max_act = 0;                // largest per-row activation (elements) between layers
};

inline int same_out(int n, int s) { return (n + s - 1) / s; }
inline int same_pad_before(int n, int k, int s) {
    int total = (same_out(n, s) - 1) * s + k - n;
    if (total < 0) total = 0;
    return total / 2;
}

// Returns SEED_OK and fills `p`, or an error status with a message in `err`.
inline seed_status_t make_plan(const seed_arch_t* a, Plan& p, std::string& err) {
    char msg[256];
    auto fail = [&](seed_status_t st, const char* m) { err = m; return st; };
    if (!a) return fail(SEED_ERR_INVALID_ARG, "arch is NULL");
    if (a->struct_size != sizeof(seed_arch_t)) {
        snprintf(msg, sizeof msg, "arch.struct_size is %u, this library expects %zu", a->struct_size,
                 sizeof(seed_arch_t));
        return fail(SEED_ERR_INVALID_ARG, msg);
    }
    if (a->obs_h <= 0 || a->obs_w <= 0 || a->obs_c <= 0) return fail(SEED_ERR_INVALID_ARG, "observation extent must be positive");
    if (a->obs_h > 4096 || a->obs_w > 4096 || a->obs_c > 1024) return fail(SEED_ERR_INVALID_ARG, "observation extent too large");
    if (a->fc_units <= 0 || a->fc_units > 8192) return fail(SEED_ERR_INVALID_ARG, "fc_units out of range");
    if (a->lstm_units < 0 || a->lstm_units > 8192) return fail(SEED_ERR_INVALID_ARG, "lstm_units out of range");
    if (a->num_actions <= 0 || a->num_actions > SEED_MAX_ACTIONS) return fail(SEED_ERR_INVALID_ARG, "num_actions must be in 1..64");
    if (a->head != SEED_HEAD_POLICY_VALUE && a->head != SEED_HEAD_DUELING_Q) return fail(SEED_ERR_INVALID_ARG, "unknown head");
    if (a->head == SEED_HEAD_DUELING_Q && (a->head_hidden <= 0 || a->head_hidden > 8192))
        return fail(SEED_ERR_INVALID_ARG, "dueling head needs head_hidden in 1..8192");
    if (a->select != SEED_SELECT_GREEDY && a->select != SEED_SELECT_GUMBEL) return fail(SEED_ERR_INVALID_ARG, "unknown select");
    if (a->precision != SEED_PRECISION_FP32 && a->precision != SEED_PRECISION_BF16) return fail(SEED_ERR_INVALID_ARG, "unknown precision");
    if (a->max_batch <= 0 || a->max_batch > (1 << 20)) return fail(SEED_ERR_INVALID_ARG, "max_batch must be in 1..2^20");

    p = Plan{};
    p.arch = *a;
    size_t off = 0;
    int H = a->obs_h, W = a->obs_w, C = a->obs_c;
    p.max_act = (size_t)H * W * C;
    auto bump = [&](size_t n) { if (n > p.max_act) p.max_act = n; };

    if (a->torso == SEED_TORSO_CONV_STACK) {
        if (a->n_conv < 1 || a->n_conv > SEED_MAX_LAYERS) return fail(SEED_ERR_INVALID_ARG, "n_conv must be in 1..4");
        for (int l = 0; l < a->n_conv; ++l) {
            int k = a->conv_k[l], s = a->conv_stride[l], co = a->conv_ch[l];
            if (k <= 0 || k > 16 || s <= 0 || s > k || co <= 0 || co > 1024)
                return fail(SEED_ERR_INVALID_ARG, "conv layer: need 1<=k<=16, 1<=stride<=k, 1<=channels<=1024");
            if (H < k || W < k) return fail(SEED_ERR_INVALID_ARG, "conv kernel larger than its input");
            ConvLayer c{};
            c.H = H; c.W = W; c.Cin = C; c.k = k; c.stride = s; c.pad = 0;
            c.OH = (H - k) / s + 1; c.OW = (W - k) / s + 1; c.Cout = co;
            c.w_off = off; off += (size_t)k * k * C * co;
            c.b_off = off; off += co;
            p.convs.push_back(c);
            H = c.OH; W = c.OW; C = co;
            bump((size_t)H * W * C);
        }
    } else if (a->torso == SEED_TORSO_RESNET) {
        if (a->n_sections < 1 || a->n_sections > SEED_MAX_LAYERS) return fail(SEED_ERR_INVALID_ARG, "n_sections must be in 1..4");
        for (int s = 0; s < a->n_sections; ++s) {
            int co = a->section_ch[s];
            if (co <= 0 || co > 1024) return fail(SEED_ERR_INVALID_ARG, "section channels must be in 1..1024");
            Section sec{};
            ConvLayer& c = sec.conv0;
            c.H = H; c.W = W; c.Cin = C; c.k = 3; c.stride = 1; c.pad = 1; c.OH = H; c.OW = W; c.Cout = co;
            c.w_off = off; off += (size_t)9 * C * co;
            c.b_off = off; off += co;
            bump((size_t)H * W * co);
            sec.PH = same_out(H, 2); sec.PW = same_out(W, 2);
            sec.pool_pad_h = same_pad_before(H, 3, 2); sec.pool_pad_w = same_pad_before(W, 3, 2);
            H = sec.PH; W = sec.PW; C = co;
            for (int j = 0; j < 4; ++j) {
                ConvLayer& b = sec.block[j];
                b.H = H; b.W = W; b.Cin = C; b.k = 3; b.stride = 1; b.pad = 1; b.OH = H; b.OW = W; b.Cout = C;
                b.w_off = off; off += (size_t)9 * C * C;
                b.b_off = off; off += C;
            }
            p.sections.push_back(sec);
        }
    } else {
        return fail(SEED_ERR_INVALID_ARG, "unknown torso");
    }
    p.feat_h = H; p.feat_w = W; p.feat_c = C;
    p.flat = (size_t)H * W * C;
    p.fc_w = off; off += p.flat * a->fc_units;
    p.fc_b = off; off += a->fc_units;
    p.core = a->fc_units;
    if (a->lstm_units > 0) {
        size_t rows = (size_t)a->fc_units + a->num_actions + 1 + a->lstm_units;
        p.lstm_w = off; off += rows * 4 * a->lstm_units;
        p.lstm_b = off; off += (size_t)4 * a->lstm_units;
        p.core = a->lstm_units;
    }
    int A = a->num_actions;
    if (a->head == SEED_HEAD_POLICY_VALUE) {
        p.pol_w = off; off += (size_t)p.core * A;
        p.pol_b = off; off += A;
        p.val_w = off; off += p.core;
        p.val_b = off; off += 1;
    } else {
        int hid = a->head_hidden;
        p.v1_w = off; off += (size_t)p.core * hid;
        p.v1_b = off; off += hid;
        p.v2_w = off; off += hid;
        p.v2_b = off; off += 1;
        p.a1_w = off; off += (size_t)p.core * hid;
        p.a1_b = off; off += hid;
        p.a2_w = off; off += (size_t)hid * A;
        p.a2_b = off; off += A;
    }
    p.n_weights = off;
    return SEED_OK;
}

}  // namespace seedinf
