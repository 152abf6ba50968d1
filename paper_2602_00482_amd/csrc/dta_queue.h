// Work queues for launches that run as a fixed set of resident blocks: one
// queue per kv head, an int counter in device memory that says how many of the
// head's items (numbered longest first) have been handed out.  A block drains
// the queue of its home head, blockIdx.x % n_queues, first: blocks are placed
// round-robin over the 8 XCDs, so that keeps a head's rows in the L2 of the XCD
// the block runs on; when that queue is empty it takes from the next heads'
// queues, so that XCDs that run faster, or finish early, take over work from the
// others.  Which block computes which item never changes a result.
#pragma once

#include <hip/hip_runtime.h>

namespace dta {

struct ItemQueues {
  int* tickets;   // [n_queues], zero at launch
  int n_items;    // per queue
  int n_queues;
  int queue;      // the queue this block is drawing from
  int pending;    // thread 0: ticket drawn ahead by prefetch()

  __device__ __forceinline__ void init(int* t, int items, int queues) {
    tickets = t; n_items = items; n_queues = queues;
    queue = blockIdx.x % queues;
    pending = 0;
  }
  // Starts the draw of the next ticket; to be called by every thread some time
  // before draw(.., true), so that the atomic's round trip is covered by other
  // work (the stores at the end of an item).
  __device__ __forceinline__ void prefetch() {
    if (threadIdx.x == 0) pending = atomicAdd(&tickets[queue], 1);
  }
  // Called by every thread of the block at the same point; `slot` = two ints of
  // LDS that nothing else touches between the two barriers in here and the next
  // barrier of the caller.  Returns false when all queues are empty.  Every
  // atomic either hands out an item or moves on to the next of n_queues queues,
  // so the loop ends.
  __device__ __forceinline__ bool draw(int* slot, int& item, int& head, bool have_pending) {
    __syncthreads();   // everyone is done with the previous item's LDS data and with slot
    if (threadIdx.x == 0) {
      int it = -1, q = queue;
      int t = have_pending ? pending : atomicAdd(&tickets[q], 1);
      for (int tries = 1;; ++tries) {
        if (t < n_items) { it = t; break; }
        if (tries == n_queues) break;
        q = q + 1 == n_queues ? 0 : q + 1;
        t = atomicAdd(&tickets[q], 1);
      }
      slot[0] = it;
      slot[1] = q;
    }
    __syncthreads();
    item = __builtin_amdgcn_readfirstlane(slot[0]);
    head = __builtin_amdgcn_readfirstlane(slot[1]);
    queue = head;
    return item >= 0;
  }
};

}  // namespace dta
