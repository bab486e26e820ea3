// Pinned staging ring of the host side: small host-to-device uploads (page tables, job lists, parameter blocks of a
// ragged batch) are copied into it and read from there by work enqueued on the cache's stream.  The ring is cut
// into segments; when the write position leaves a segment, a marker is recorded on the stream behind everything
// that reads the segment, and a segment is written again only after its marker has been reached.  The host
// therefore never waits for the whole stream: it blocks only if it has run a full ring ahead of the device.
//
// The marker mechanism is a template parameter so that the bookkeeping can be exercised on the CPU with a fake.
//   struct Backend { bool record(int segment);   // enqueue a marker behind the work issued so far
//                    bool wait(int segment); };  // block until the marker of that segment has been reached
#ifndef KVQ_RING_H
#define KVQ_RING_H

#include <stdint.h>

template <class Backend, int N_SEGMENTS>
class KvqStagingRing {
public:
    // segment_bytes: multiple of 256.  The ring spans N_SEGMENTS * segment_bytes bytes.
    void init(uint64_t segment_bytes) {
        seg_bytes_ = segment_bytes;
        cur_ = 0;
        pos_ = 0;
        for (int i = 0; i < N_SEGMENTS; ++i) pending_[i] = false;
    }
    uint64_t segment_bytes() const { return seg_bytes_; }
    uint64_t total_bytes() const { return seg_bytes_ * N_SEGMENTS; }
    int waits() const { return waits_; }  // how often a reservation had to wait for the device (statistics)

    // Reserves `bytes` (<= segment_bytes) at an offset that is a multiple of `align` (a power of two <= 256) and
    // returns the offset into the ring, or -1 if the request is too large or a marker call failed.
    int64_t reserve(Backend& be, uint64_t bytes, uint64_t align) {
        if (bytes == 0 || bytes > seg_bytes_) return -1;
        uint64_t at = (pos_ + align - 1) & ~(align - 1);
        if (at + bytes > seg_bytes_) {
            // leave the segment: everything enqueued so far may read it, the marker goes behind all of that
            if (!be.record(cur_)) return -1;
            pending_[cur_] = true;
            cur_ = (cur_ + 1) % N_SEGMENTS;
            if (pending_[cur_]) {
                if (!be.wait(cur_)) return -1;
                pending_[cur_] = false;
                ++waits_;
            }
            at = 0;
        }
        pos_ = at + bytes;
        return (int64_t)((uint64_t)cur_ * seg_bytes_ + at);
    }

private:
    uint64_t seg_bytes_ = 0, pos_ = 0;
    int cur_ = 0, waits_ = 0;
    bool pending_[N_SEGMENTS];
};

#endif
