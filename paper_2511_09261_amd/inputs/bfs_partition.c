/* Seeded BFS region growing: the partitioner that makes the part_id input array
 * of the synthetic workloads.  It is an input generator only (the paper uses
 * Louvain communities, Sec. 3.1; the workloads here fix the partition ids as an
 * input), and contains nothing of the training method.
 *
 * Rule.  cap = ceil(n / P).  Region k starts from roots[k].  Regions take turns
 * in order k = 0..P-1; on its turn a region pops one node from its FIFO and
 * claims that node's unassigned neighbours in ascending id order until the
 * region holds cap nodes.  When no region can advance (every FIFO empty or
 * region full) the smallest unassigned id goes to the currently smallest region
 * (ties: lowest k) and becomes a new BFS root there.
 *
 * Build: gcc -O2 -shared -fPIC bfs_partition.c -o libbfs_partition.so
 */
#include <stdint.h>
#include <stdlib.h>

int bfs_region_growing(int64_t n, const int64_t* rowptr, const int32_t* col,
                       int32_t P, const int32_t* roots, int32_t* part) {
  if (n < 0 || P < 1 || (int64_t)P > (n > 0 ? n : 1)) return -1;
  if (n == 0) return 0;
  const int64_t cap = (n + P - 1) / P;
  /* one FIFO per region, each of capacity cap, in one allocation */
  int32_t* fifo = (int32_t*)malloc((size_t)P * (size_t)cap * sizeof(int32_t));
  int64_t* head = (int64_t*)calloc((size_t)P, sizeof(int64_t));
  int64_t* tail = (int64_t*)calloc((size_t)P, sizeof(int64_t));
  int64_t* size = (int64_t*)calloc((size_t)P, sizeof(int64_t));
  if (!fifo || !head || !tail || !size) { free(fifo); free(head); free(tail); free(size); return -2; }
  for (int64_t i = 0; i < n; ++i) part[i] = -1;
  for (int32_t k = 0; k < P; ++k) {
    int32_t r = roots[k];
    if (r < 0 || r >= n || part[r] != -1) { free(fifo); free(head); free(tail); free(size); return -3; }
    part[r] = k;
    fifo[(int64_t)k * cap + tail[k]++] = r;
    size[k] = 1;
  }
  int64_t assigned = P;
  int64_t next_free = 0; /* every id below next_free is assigned */
  while (assigned < n) {
    int progressed = 0;
    for (int32_t k = 0; k < P; ++k) {
      if (head[k] == tail[k]) continue;
      if (size[k] >= cap) { head[k] = tail[k]; continue; }
      int32_t u = fifo[(int64_t)k * cap + head[k]++];
      progressed = 1;
      for (int64_t e = rowptr[u]; e < rowptr[u + 1] && size[k] < cap; ++e) {
        int32_t v = col[e];
        if (part[v] == -1) {
          part[v] = k;
          fifo[(int64_t)k * cap + tail[k]++] = v;
          ++size[k];
          ++assigned;
        }
      }
    }
    if (progressed || assigned >= n) continue;
    while (next_free < n && part[next_free] != -1) ++next_free;
    if (next_free >= n) break;
    int32_t best = 0;
    for (int32_t k = 1; k < P; ++k) if (size[k] < size[best]) best = k;
    part[next_free] = best;
    fifo[(int64_t)best * cap + tail[best]++] = (int32_t)next_free;
    ++size[best];
    ++assigned;
  }
  free(fifo); free(head); free(tail); free(size);
  return 0;
}
