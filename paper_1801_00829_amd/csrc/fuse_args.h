/* Kernel argument block shared by the host launcher and the hipRTC-compiled
 * skeletons (this file's text is prepended to every generated source). */
#ifndef FUSE_ARGS_H
#define FUSE_ARGS_H

#define FUSE_MAX_SIDES 8
#define FUSE_MAX_AGGS 16
#ifndef FUSE_MAX_K
#define FUSE_MAX_K 16
#endif

typedef struct {
    const double *x;                          /* dense main input, or CSR values      */
    const int *colidx;                        /* CSR column indices                   */
    const void *rowptr;                       /* CSR row offsets (int32 or int64)     */
    const double *side[FUSE_MAX_SIDES];       /* side inputs (device)                 */
    long long side_ld[FUSE_MAX_SIDES];        /* leading dimension / row stride       */
    double side_scalar[FUSE_MAX_SIDES];       /* scalar sides                         */
    const double *u, *v;                      /* Outer factors                        */
    long long ldu, ldv;
    long long m, n, ld, nnz;                  /* shape of the main input              */
    double *out;
    double *partials;                         /* workspace: per-block partial sums    */
    unsigned int *ticket;                     /* workspace: zeroed arrival counter    */
    int rank;                                 /* Outer: columns of U and V            */
    int npanels;                              /* Outer: column panels of V (0: none)  */
    void *panel_ptr;                          /* Outer workspace: per panel and row, the first stored cell at or
                                                 after the panel's first column ((npanels+1) x m offsets)         */
    int panel_w;                              /* Outer: columns per panel             */
    int pad_;
    const int *side_ci[FUSE_MAX_SIDES];       /* sparse side inputs: column indices (values in side[], stored  */
    const void *side_rp[FUSE_MAX_SIDES];      /*   cells in side_ld[]), row offsets (int32 or int64)           */
} fuse_kargs;

#endif
