// The training controller's arithmetic (host side): the sweep schedule of the chunks, the length of a
// super-epoch and the decision when to switch partitions early, fed by the step statistics the device writes.
#include "common.h"

#include <new>

struct grp_controller_s {
    int32_t n_chunks = 1;
    int64_t epochs_per_super_epoch = 1;
    double threshold = 1.0;
    int64_t patience = 0;
    int64_t super_epoch = 0, epochs_in_super_epoch = 0, over = 0;
};

extern "C" int32_t grp_sweep_chunk(int32_t worker, int64_t super_epoch, int32_t n_chunks) {
    if (n_chunks < 1 || worker < 0 || worker >= n_chunks || super_epoch < 0) return -1;
    if (n_chunks == 1) return 0;
    const int64_t t = super_epoch % (n_chunks - 1);        // the cycle of c - 1 super-epochs repeats
    return (int32_t)((worker + 1 + t) % n_chunks);
}

extern "C" int64_t grp_super_epoch_epochs(int64_t total_epochs, int32_t n_chunks) {
    if (total_epochs < 0 || n_chunks < 1) return -1;
    const int64_t cycle = n_chunks > 1 ? n_chunks - 1 : 1;
    const int64_t e = (total_epochs + cycle - 1) / cycle;
    return e > 1 ? e : 1;
}

extern "C" grp_status grp_controller_create(int64_t total_epochs, int32_t n_chunks, double threshold, int64_t patience,
                                            grp_controller_t** out) {
    if (!out) return grp::fail(GRP_EINVAL, "grp_controller_create: out is null");
    *out = nullptr;
    if (total_epochs < 0 || n_chunks < 1 || patience < 1 || !(threshold == threshold))
        return grp::fail(GRP_EINVAL, "grp_controller_create: total_epochs >= 0, n_chunks >= 1, patience >= 1 and a threshold are needed");
    grp_controller_t* c = new (std::nothrow) grp_controller_t();
    if (!c) return grp::fail(GRP_ENOMEM, "host allocation failed");
    c->n_chunks = n_chunks;
    c->epochs_per_super_epoch = grp_super_epoch_epochs(total_epochs, n_chunks);
    c->threshold = threshold;
    c->patience = patience;
    *out = c;
    return GRP_OK;
}

static grp_status observe_deficit(grp_controller_t* ctl, double mean_c) {
    const double deficit = 1.0 - mean_c;
    ctl->over = deficit > ctl->threshold ? ctl->over + 1 : 0;
    return GRP_OK;
}

extern "C" grp_status grp_controller_observe(grp_controller_t* ctl, const float* c_hat, int32_t m) {
    if (!ctl || !c_hat || m < 1) return grp::fail(GRP_EINVAL, "grp_controller_observe: bad arguments");
    double sum = 0.0;
    for (int32_t i = 0; i < m; ++i) sum += (double)c_hat[i];
    return observe_deficit(ctl, sum / m);
}

extern "C" grp_status grp_controller_observe_stats(grp_controller_t* ctl, const grp_step_stats* stats, int32_t m) {
    if (!ctl || !stats || m < 1) return grp::fail(GRP_EINVAL, "grp_controller_observe_stats: bad arguments");
    double sum = 0.0;
    for (int32_t i = 0; i < m; ++i) sum += stats[i].S > 0 ? stats[i].sum_ratio / (double)stats[i].S : 1.0;
    return observe_deficit(ctl, sum / m);
}

extern "C" grp_status grp_controller_end_epoch(grp_controller_t* ctl, int32_t* switched) {
    if (!ctl || !switched) return grp::fail(GRP_EINVAL, "grp_controller_end_epoch: bad arguments");
    ctl->epochs_in_super_epoch += 1;
    *switched = 0;
    if (ctl->epochs_in_super_epoch >= ctl->epochs_per_super_epoch || ctl->over >= ctl->patience) {
        ctl->super_epoch += 1;
        ctl->epochs_in_super_epoch = 0;
        ctl->over = 0;
        *switched = 1;
    }
    return GRP_OK;
}

extern "C" grp_status grp_controller_state(const grp_controller_t* ctl, int64_t* super_epoch, int64_t* epochs_per_super_epoch) {
    if (!ctl) return grp::fail(GRP_EINVAL, "grp_controller_state: null controller");
    if (super_epoch) *super_epoch = ctl->super_epoch;
    if (epochs_per_super_epoch) *epochs_per_super_epoch = ctl->epochs_per_super_epoch;
    return GRP_OK;
}

extern "C" grp_status grp_controller_destroy(grp_controller_t* ctl) {
    delete ctl;
    return GRP_OK;
}
