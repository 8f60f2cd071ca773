// Test-only C wrapper around the library's host-side protocol state machine
// (paper_2506_04531_amd/csrc/protocol.hpp), so that its decisions can be checked without a GPU.
#include "../../paper_2506_04531_amd/csrc/protocol.hpp"

using halos::LpsProtocol;

extern "C" {
void *proto_new(int n_workers, int K) { return new LpsProtocol(n_workers, K); }
void proto_free(void *p) { delete (LpsProtocol *)p; }
int proto_set_K(void *p, int K) { return ((LpsProtocol *)p)->set_K(K); }
int proto_push_delta(void *p, int worker) {
    LpsProtocol *s = (LpsProtocol *)p;
    int rc = s->can_push_delta(worker);
    if (rc == halos::PROTO_OK) s->push_delta(worker);
    return rc;
}
int proto_push_global(void *p) {
    LpsProtocol *s = (LpsProtocol *)p;
    int rc = s->can_push_global();
    if (rc == halos::PROTO_OK) s->push_global();
    return rc;
}
// out = {kind, worker, accumulate, freezes, t, t_last}
int proto_step(void *p, long long *out) {
    LpsProtocol *s = (LpsProtocol *)p;
    halos::QueueItem h = s->head();
    out[0] = h.kind; out[1] = h.worker; out[2] = 0; out[3] = 0;
    if (h.kind == halos::ITEM_DELTA) {
        halos::UpdateOutcome o = s->preview_update();
        out[2] = o.accumulate; out[3] = o.freezes;
        s->commit_update();
    } else if (h.kind == halos::ITEM_GLOBAL) {
        s->commit_merge();
    }
    out[4] = s->t(); out[5] = s->t_last();
    return 0;
}
// averaged step over the first `count` items: -1 if they are not all deltas; out as in proto_step (worker = the last sender)
int proto_step_average(void *p, int count, long long *out) {
    LpsProtocol *s = (LpsProtocol *)p;
    if (!s->head_is_deltas(count)) return -1;
    halos::UpdateOutcome o = s->preview_update();
    out[0] = halos::ITEM_DELTA; out[1] = s->item(count - 1).worker; out[2] = o.accumulate; out[3] = o.freezes;
    s->commit_average(count);
    out[4] = s->t(); out[5] = s->t_last();
    return 0;
}
int proto_consume(void *p) {
    LpsProtocol *s = (LpsProtocol *)p;
    int rc = s->can_consume();
    if (rc == halos::PROTO_OK) s->consume();
    return rc;
}
// momentum cycle of the delayed rule
void *cycle_new() { return new halos::MomentumCycle; }
void cycle_free(void *p) { delete (halos::MomentumCycle *)p; }
int cycle_set_d(void *p, int d) { return ((halos::MomentumCycle *)p)->set_d(d); }
int cycle_next(void *p) { return ((halos::MomentumCycle *)p)->next(); }
void cycle_commit(void *p) { ((halos::MomentumCycle *)p)->commit(); }
int cycle_seen(void *p) { return ((halos::MomentumCycle *)p)->seen(); }
int cycle_d(void *p) { return ((halos::MomentumCycle *)p)->d(); }
int proto_phase(void *p) { return ((LpsProtocol *)p)->phase(); }
int proto_queued(void *p) { return ((LpsProtocol *)p)->queued(); }
}
