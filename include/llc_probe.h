/* llc_probe.h -- machine probes used by the benchmark (libllc_probe.so; not part of the sampler).
 *
 * llc_probe_run(which, reps, &result, &clock_ghz) runs `reps` launches of one probe kernel on the
 * current device (after as many warm-up launches), on the default stream, synchronously; it
 * allocates and frees its own buffers.  result: operations (or operation pairs, 32-bit words,
 * bytes) per second; clock_ghz (not for READ and COPY): shader-clock cycles of the last launch's first
 * wavefront divided by the same span on the constant 100 MHz counter, in GHz.  Returns 0, or
 * -1 on a bad argument or a HIP error.
 */
#ifndef LLC_PROBE_H_
#define LLC_PROBE_H_

#ifdef __cplusplus
extern "C" {
#endif

enum {
  LLC_PROBE_FMA = 0,     /* fp32 fused multiply-adds per second                               */
  LLC_PROBE_MAD_XOR = 1, /* (32x32->64 product, xor) pairs per second: a Philox round's core   */
  LLC_PROBE_XOR3 = 2,    /* three-input xors per second                                        */
  LLC_PROBE_PHILOX = 3,  /* 32-bit words of full Philox4x32-10 blocks per second               */
  LLC_PROBE_READ = 4,    /* bytes per second of a streaming read of 4 GiB                      */
  LLC_PROBE_COPY = 5,    /* bytes read + written per second of a 4 GiB copy                    */
  LLC_PROBE_PHILOX_READ = 6 /* bytes per second of a 4 GiB streaming read with one Philox block
                               generated per 8 bytes read (generator and memory together)       */
};

int llc_probe_run(int which, int reps, double *result, double *clock_ghz);

#ifdef __cplusplus
}
#endif
#endif /* LLC_PROBE_H_ */
