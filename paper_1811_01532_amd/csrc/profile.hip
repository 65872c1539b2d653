// wap_profile_layer: the measured t_c(l, b) table -- forward / data-gradient / weight-gradient time
// of one layer at each per-GPU minibatch b, with algorithmic FLOPs and bytes, TFLOP/s against the
// bf16 MFMA peak and GB/s against the HBM peak.  This is the input the workload analysis unit of
// Section 3.2.1 needs to evaluate Eq. 1 for every candidate GPU count d (per-GPU minibatch B/d).
#include <algorithm>
#include <cmath>
#include <vector>

#include "wap_internal.h"

using namespace wap;

namespace {

constexpr double kProfileSampleUs = 100.0;   // samples shorter than this bracket several launches
constexpr double kLaunchBoundFactor = 4.0;   // slower than 4x both roofs: class 2 (launch / occupancy)

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
    size_t x, w, y, yo, dx, dw, ws, total;
    size_t x_elems, w_elems, y_elems;
    size_t ws_bytes;
};

struct Passes {
    GemmGeom gf, gd;
    GemmPlan pf, pd;
    WgradGeom gw;
    WgradPlan pw;
};

int make_passes(int kind, const void* desc, int mb, Passes* ps, Layout* lay) {
    size_t xe, we, ye;
    if (kind == 0) {
        wap_conv_desc d = *reinterpret_cast<const wap_conv_desc*>(desc);
        d.N = mb;
        int rc = validate_conv(&d);
        if (rc != WAP_OK) return rc;
        ps->gf = geom_conv_fwd(d);
        ps->gd = geom_conv_dgrad(d);
        ps->gw = geom_conv_wgrad(d);
        xe = (size_t)d.N * d.H * d.W * d.C;
        we = (size_t)d.K * d.R * d.S * d.C;
        ye = (size_t)ps->gf.M * d.K;
    } else if (kind == 1) {
        wap_fc_desc d = *reinterpret_cast<const wap_fc_desc*>(desc);
        d.B = mb;
        int rc = validate_fc(&d);
        if (rc != WAP_OK) return rc;
        ps->gf = geom_fc_fwd(d);
        ps->gd = geom_fc_dx(d);
        ps->gw = geom_fc_dw(d);
        xe = (size_t)d.B * d.in_features;
        we = (size_t)d.in_features * d.out_features;
        ye = (size_t)d.B * d.out_features;
    } else {
        return set_error(WAP_EINVAL, "profile: kind must be 0 (conv) or 1 (fc)");
    }
    ps->pf = plan_fwd_like(ps->gf, false);
    ps->pd = plan_fwd_like(ps->gd, true);
    ps->pw = plan_wgrad(ps->gw);
    lay->x_elems = xe; lay->w_elems = we; lay->y_elems = ye;
    lay->ws_bytes = std::max(ps->pf.ws_bytes, std::max(ps->pd.ws_bytes, ps->pw.ws_bytes));
    size_t o = 0;
    lay->x = o; o = align_up(o + xe * 2, 256);
    lay->w = o; o = align_up(o + we * 2, 256);
    lay->y = o; o = align_up(o + ye * 2, 256);
    lay->yo = o; o = align_up(o + ye * 2, 256);
    lay->dx = o; o = align_up(o + xe * 2, 256);
    lay->dw = o; o = align_up(o + we * 4, 256);
    lay->ws = o; o = align_up(o + lay->ws_bytes, 256);
    lay->total = o;
    return WAP_OK;
}

}  // namespace

extern "C" {

int wap_profile_scratch_bytes(int kind, const void* desc, const int32_t* minibatches, int32_t n_mb,
                              size_t* bytes_out) {
    if (!desc || !minibatches || !bytes_out || n_mb < 1) return set_error(WAP_EINVAL, "profile: bad argument");
    size_t need = 0;
    for (int i = 0; i < n_mb; ++i) {
        Passes ps;
        Layout lay;
        int rc = make_passes(kind, desc, minibatches[i], &ps, &lay);
        if (rc != WAP_OK) return rc;
        need = std::max(need, lay.total);
    }
    *bytes_out = need;
    return WAP_OK;
}

int wap_profile_layer(int kind, const void* desc, const int32_t* minibatches, int32_t n_mb, int32_t warmup,
                      int32_t iters, void* scratch, size_t scratch_bytes, void* stream,
                      wap_profile_row* rows_out, int32_t rows_cap, int32_t* rows_written) {
    if (!desc || !minibatches || !rows_out || !rows_written || n_mb < 1 || iters < 1 || warmup < 0)
        return set_error(WAP_EINVAL, "profile: bad argument");
    if (rows_cap < 3 * n_mb) return set_error(WAP_EINVAL, "profile: rows_cap %d below 3*n_mb", rows_cap);
    if (!scratch || (reinterpret_cast<uintptr_t>(scratch) & 255u))
        return set_error(WAP_EINVAL, "profile: scratch must be non-NULL and 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    // One event per sample boundary, all recorded without a host synchronisation in between: the queue never runs
    // dry, so the host's launch latency is not part of a sample (a sample that starts on an idle queue is stamped
    // before the host has finished enqueuing the pass).  Short passes are timed as `reps` back-to-back launches per
    // sample, so that the few microseconds an event record costs between two kernels stay small against the sample.
    std::vector<hipEvent_t> ev((size_t)iters + 1, nullptr);
    for (auto& e : ev)
        if (hipEventCreate(&e) != hipSuccess) {
            for (auto& f : ev)
                if (f) (void)hipEventDestroy(f);
            return set_error(WAP_EHIP, "profile: hipEventCreate failed");
        }
    int rc = WAP_OK;
    int nrows = 0;
    unsigned char* base = (unsigned char*)scratch;
    std::vector<float> t((size_t)iters);
    for (int i = 0; i < n_mb && rc == WAP_OK; ++i) {
        Passes ps;
        Layout lay;
        rc = make_passes(kind, desc, minibatches[i], &ps, &lay);
        if (rc != WAP_OK) break;
        if (lay.total > scratch_bytes) {
            rc = set_error(WAP_EWORKSPACE, "profile: scratch has %zu bytes, %zu needed at minibatch %d", scratch_bytes,
                           lay.total, minibatches[i]);
            break;
        }
        bf16_t* x = (bf16_t*)(base + lay.x);
        bf16_t* w = (bf16_t*)(base + lay.w);
        bf16_t* y = (bf16_t*)(base + lay.y);
        bf16_t* yo = (bf16_t*)(base + lay.yo);
        bf16_t* dx = (bf16_t*)(base + lay.dx);
        float* dw = (float*)(base + lay.dw);
        void* ws = base + lay.ws;
        if ((rc = launch_fill_bf16(x, lay.x_elems, 1u, st)) != WAP_OK) break;
        if ((rc = launch_fill_bf16(w, lay.w_elems, 2u, st)) != WAP_OK) break;
        if ((rc = launch_fill_bf16(y, lay.y_elems, 3u, st)) != WAP_OK) break;
        const double flops = 2.0 * (double)ps.gf.M * ps.gf.Ncols * ps.gf.Kred;
        const double bytes_pass[3] = {
            2.0 * (lay.x_elems + lay.w_elems + lay.y_elems),
            2.0 * (lay.y_elems + lay.w_elems + lay.x_elems),
            2.0 * (lay.x_elems + lay.y_elems) + 4.0 * lay.w_elems,
        };
        for (int pass = 0; pass < 3 && rc == WAP_OK; ++pass) {
            auto run = [&]() -> int {
                if (pass == 0) return launch_fwd_like(ps.gf, false, ps.pf, x, w, nullptr, true, yo, ws, st);
                if (pass == 1) return launch_fwd_like(ps.gd, true, ps.pd, y, w, nullptr, false, dx, ws, st);
                return launch_wgrad(ps.gw, ps.pw, x, y, dw, ws, st);
            };
            // warm-up (at least one launch: its time sizes `reps`)
            const int nwarm = warmup > 0 ? warmup : 1;
            (void)hipEventRecord(ev[0], st);
            for (int k = 0; k < nwarm && rc == WAP_OK; ++k) rc = run();
            (void)hipEventRecord(ev[1], st);
            if (rc != WAP_OK) break;
            if (hipEventSynchronize(ev[1]) != hipSuccess) { rc = set_error(WAP_EHIP, "profile: event sync failed"); break; }
            float wms = 0.f;
            (void)hipEventElapsedTime(&wms, ev[0], ev[1]);
            const double warm_us = (double)wms * 1000.0 / nwarm;
            int reps = 1;
            if (warm_us < kProfileSampleUs) reps = (int)std::min(8.0, std::ceil(kProfileSampleUs / std::max(warm_us, 1.0)));
            (void)hipEventRecord(ev[0], st);
            for (int k = 0; k < iters && rc == WAP_OK; ++k) {
                for (int q = 0; q < reps && rc == WAP_OK; ++q) rc = run();
                (void)hipEventRecord(ev[(size_t)k + 1], st);
            }
            if (rc != WAP_OK) break;
            if (hipEventSynchronize(ev[(size_t)iters]) != hipSuccess) { rc = set_error(WAP_EHIP, "profile: event sync failed"); break; }
            for (int k = 0; k < iters; ++k) {
                float ms = 0.f;
                (void)hipEventElapsedTime(&ms, ev[(size_t)k], ev[(size_t)k + 1]);
                t[k] = ms * 1000.f / (float)reps;
            }
            std::vector<float> s(t);
            std::sort(s.begin(), s.end());
            wap_profile_row& r = rows_out[nrows++];
            r.pass = pass;
            r.minibatch = minibatches[i];
            r.flops = flops;
            r.alg_bytes = bytes_pass[pass];
            r.time_us_median = s[s.size() / 2];
            r.time_us_min = s[0];
            r.tflops = flops / (r.time_us_median * 1e-6) / 1e12;
            r.frac_of_bf16_peak = r.tflops / kPeakBf16Tflops;
            r.gbytes_per_s = r.alg_bytes / (r.time_us_median * 1e-6) / 1e9;
            r.frac_of_hbm_peak = r.gbytes_per_s / kPeakHbmGBs;
            // Which roof the pass sits under: the side of the ridge its arithmetic intensity falls on, unless the
            // measured time is more than kLaunchBoundFactor times the time of BOTH roofs -- then neither the matrix
            // pipes nor HBM explain it and the pass is bound by launch overhead / too few work-groups for the chip,
            // the small-minibatch regime of Section 2.2.
            const double t_mfma_us = flops / (kPeakBf16Tflops * 1e12) * 1e6;
            const double t_hbm_us = r.alg_bytes / (kPeakHbmGBs * 1e9) * 1e6;
            r.bound = (t_mfma_us >= t_hbm_us) ? 0 : 1;
            if (r.time_us_median > kLaunchBoundFactor * std::max(t_mfma_us, t_hbm_us)) r.bound = 2;
            r.reps_per_sample = reps;
        }
    }
    for (auto& e : ev) (void)hipEventDestroy(e);
    *rows_written = nrows;
    return rc;
}

}  // extern "C"
