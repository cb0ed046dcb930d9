/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * Plain, slow, single-threaded CPU statement of what the FastGS rasterizer hot path
 * computes, written from the paper's equations.  Only the test-suite, the smoke check and
 * the benchmark's CPU-baseline leg may call it.  It shares no code with the HIP path.
 *
 * This body is compiled twice (see fastgs_oracle.c): once with REAL = float, where every
 * value that feeds an integer decision follows the pinned fp32 operation order described
 * next to each step (plain IEEE + - * / sqrt, left to right as written, fused multiply-add
 * only where FMA() is spelled out, no contraction), and once with REAL = double for the
 * finite-difference checks, where EXPNEG is the C library's exp().
 *
 * Sums over pixels (gradients, image statistics) are kept in double in both builds.
 *
 * Notation follows the paper: mu (mean), s (scale), r/q (rotation quaternion), sigma
 * (opacity), c (SH colour coefficients), W (viewing transform, here Rc,t0), J (Jacobian of
 * the projective map), Sigma_3D / Sigma_2D, alpha_i, T (transmittance), C(p).
 */

/* camera array layout: fx fy cx cy R[9] (row-major, x_cam = R x_world + t) t[3]          */
/* config array layout: z_near lowpass alpha_min alpha_max T_min bg[3] jclamp compact_box cb_beta */
#define CAM_FX(c) ((c)[0])
#define CAM_FY(c) ((c)[1])
#define CAM_CX(c) ((c)[2])
#define CAM_CY(c) ((c)[3])
#define CAM_R(c) ((c) + 4)
#define CAM_T(c) ((c) + 13)
#define CFG_ZNEAR(c) ((c)[0])
#define CFG_LOWPASS(c) ((c)[1])
#define CFG_AMIN(c) ((c)[2])
#define CFG_AMAX(c) ((c)[3])
#define CFG_TMIN(c) ((c)[4])
#define CFG_BG(c) ((c) + 5)
#define CFG_JCLAMP(c) ((c)[8])
#define CFG_CB(c) ((c)[9] != (REAL)0)
#define CFG_CB_BETA(c) ((c)[10])

/* Real spherical harmonics, bands 0..3, orthonormal on the sphere, in the textbook
 * Cartesian closed forms (no Condon-Shortley sign).  Order: (l,m) = (0,0), (1,-1), (1,0),
 * (1,1), (2,-2) ... (3,3).  Sec. 3: "view-dependent spherical harmonics", 16 x 3.          */
static void FN(sh_basis)(REAL x, REAL y, REAL z, REAL Y[16])
{
    const REAL k0 = (REAL)0.28209479177387814;  /* 1/(2 sqrt(pi))        */
    const REAL k1 = (REAL)0.4886025119029199;   /* sqrt(3/(4 pi))        */
    const REAL k2a = (REAL)1.0925484305920792;  /* sqrt(15/pi)/2         */
    const REAL k2b = (REAL)0.31539156525252005; /* sqrt(5/pi)/4          */
    const REAL k2c = (REAL)0.5462742152960396;  /* sqrt(15/pi)/4         */
    const REAL k3a = (REAL)0.5900435899266435;  /* sqrt(35/(2 pi))/4     */
    const REAL k3b = (REAL)2.890611442640554;   /* sqrt(105/pi)/2        */
    const REAL k3c = (REAL)0.4570457994644658;  /* sqrt(21/(2 pi))/4     */
    const REAL k3d = (REAL)0.3731763325901154;  /* sqrt(7/pi)/4          */
    const REAL k3e = (REAL)1.445305721320277;   /* sqrt(105/pi)/4        */
    REAL xx = x * x, yy = y * y, zz = z * z;
    Y[0] = k0;
    Y[1] = k1 * y;
    Y[2] = k1 * z;
    Y[3] = k1 * x;
    Y[4] = k2a * (x * y);
    Y[5] = k2a * (y * z);
    Y[6] = k2b * ((REAL)2 * zz - xx - yy);
    Y[7] = k2a * (x * z);
    Y[8] = k2c * (xx - yy);
    Y[9] = k3a * (y * ((REAL)3 * xx - yy));
    Y[10] = k3b * ((x * y) * z);
    Y[11] = k3c * (y * ((REAL)4 * zz - xx - yy));
    Y[12] = k3d * (z * ((REAL)2 * zz - (REAL)3 * xx - (REAL)3 * yy));
    Y[13] = k3c * (x * ((REAL)4 * zz - xx - yy));
    Y[14] = k3e * (z * (xx - yy));
    Y[15] = k3a * (x * (xx - (REAL)3 * yy));
}

/* Gradient of every basis function with respect to the (unnormalised use of the) unit
 * direction components: dY[k][0..2] = dY_k/dx, /dy, /dz of the polynomials above.          */
static void FN(sh_basis_grad)(REAL x, REAL y, REAL z, REAL dY[16][3])
{
    const REAL k1 = (REAL)0.4886025119029199, k2a = (REAL)1.0925484305920792,
               k2b = (REAL)0.31539156525252005, k2c = (REAL)0.5462742152960396,
               k3a = (REAL)0.5900435899266435, k3b = (REAL)2.890611442640554,
               k3c = (REAL)0.4570457994644658, k3d = (REAL)0.3731763325901154,
               k3e = (REAL)1.445305721320277;
    REAL xx = x * x, yy = y * y, zz = z * z;
#define SETG(k, gx, gy, gz) do { dY[k][0] = (gx); dY[k][1] = (gy); dY[k][2] = (gz); } while (0)
    SETG(0, 0, 0, 0);
    SETG(1, 0, k1, 0);
    SETG(2, 0, 0, k1);
    SETG(3, k1, 0, 0);
    SETG(4, k2a * y, k2a * x, 0);
    SETG(5, 0, k2a * z, k2a * y);
    SETG(6, k2b * (-2 * x), k2b * (-2 * y), k2b * (4 * z));
    SETG(7, k2a * z, 0, k2a * x);
    SETG(8, k2c * (2 * x), k2c * (-2 * y), 0);
    SETG(9, k3a * (6 * x * y), k3a * (3 * xx - 3 * yy), 0);
    SETG(10, k3b * (y * z), k3b * (x * z), k3b * (x * y));
    SETG(11, k3c * (-2 * x * y), k3c * (4 * zz - xx - 3 * yy), k3c * (8 * y * z));
    SETG(12, k3d * (-6 * x * z), k3d * (-6 * y * z), k3d * (6 * zz - 3 * xx - 3 * yy));
    SETG(13, k3c * (4 * zz - 3 * xx - yy), k3c * (-2 * x * y), k3c * (8 * x * z));
    SETG(14, k3e * (2 * x * z), k3e * (-2 * y * z), k3e * (xx - yy));
    SETG(15, k3a * (3 * xx - 3 * yy), k3a * (-6 * x * y), 0);
#undef SETG
}

/* Rotation matrix of a unit quaternion q = (w, x, y, z); Sec. 3 Eq. (2) uses it as R_i.    */
static void FN(quat_to_rot)(const REAL q[4], REAL R[3][3])
{
    REAL w = q[0], x = q[1], y = q[2], z = q[3];
    R[0][0] = (REAL)1 - (REAL)2 * (y * y + z * z);
    R[0][1] = (REAL)2 * (x * y - w * z);
    R[0][2] = (REAL)2 * (x * z + w * y);
    R[1][0] = (REAL)2 * (x * y + w * z);
    R[1][1] = (REAL)1 - (REAL)2 * (x * x + z * z);
    R[1][2] = (REAL)2 * (y * z - w * x);
    R[2][0] = (REAL)2 * (x * z - w * y);
    R[2][1] = (REAL)2 * (y * z + w * x);
    R[2][2] = (REAL)1 - (REAL)2 * (x * x + y * y);
}

/* Everything the projection of one Gaussian produces on the way (kept for the backward). */
typedef struct {
    int visible;
    REAL t[3];          /* camera-space mean  t = Rc mu + t0                              */
    REAL txz, tyz;      /* t_x / t_z, t_y / t_z                                           */
    REAL cxz, cyz;      /* the same, limited to +-jclamp*tan(fov/2) (used inside J only)  */
    int  xin, yin;      /* 1 where the limit is inactive                                   */
    REAL J00, J02, J11, J12;
    REAL Tm[2][3];      /* J Rc                                                            */
    REAL Rq[3][3], M[3][3], S3[3][3]; /* R_i, R_i S_i, Sigma_3D                            */
    REAL a, b, c, det;  /* Sigma_2D = [[a,b],[b,c]] (after the low-pass), its determinant  */
    REAL conic[3];      /* Sigma_2D^-1 = [[conic0, conic1],[conic1, conic2]]               */
    REAL lam_max, radius;
    REAL mx, my;        /* mu_2D                                                           */
    int  rect[4];       /* tile rectangle x0,y0,x1,y1 (half-open)                          */
    int  touched;       /* number of Gaussian-tile pairs                                    */
    REAL Q;             /* Compact Box: Mahalanobis threshold beta * 2 ln(sigma / tau_alpha) */
    REAL dir[3], len, d[3];
    REAL rgb[3]; int clamped[3];
} FN(proj);

/*
 * Compact Box (Sec. 4.4 and its supplement): the support of a Gaussian is the ellipse
 *   (p - mu_2D)^T Sigma_2D^-1 (p - mu_2D) <= Q,   Q = beta * 2 ln(sigma / tau_alpha)
 * (the supplement's equation for beta; tau_alpha is read as alpha_min), and a Gaussian-tile pair
 * exists iff the tile's closed rectangle [tile*tx, tile*tx+tile] x [tile*ty, ...] meets that ellipse,
 * i.e. iff the minimum of the quadratic form over the rectangle is <= Q.  The form is convex with its
 * minimum at mu_2D, so the minimum over the rectangle is 0 if mu_2D lies inside and otherwise sits on
 * an edge that faces mu_2D (at most one vertical and one horizontal edge); along an edge it is a
 * 1-D quadratic whose minimiser is clamped to the edge.
 * fp32 order: dxl = X0 - mx; dxr = X1 - mx; dyt = Y0 - my; dyb = Y1 - my;  vertical edge at ex:
 * dy* = min(max(-(B*ex)/C, dyt), dyb); horizontal edge at ey: dx* = min(max(-(B*ey)/A, dxl), dxr);
 * form(dx,dy) = fma(dx, fma(B+B, dy, A*dx), (C*dy)*dy).
 */
static int FN(cb_tile_hit)(REAL mx, REAL my, REAL A, REAL B, REAL C, REAL Q, int tx, int ty, int tile)
{
    REAL X0 = (REAL)(tx * tile), X1 = (REAL)(tx * tile + tile);
    REAL Y0 = (REAL)(ty * tile), Y1 = (REAL)(ty * tile + tile);
    REAL dxl = X0 - mx, dxr = X1 - mx, dyt = Y0 - my, dyb = Y1 - my;
    int in_x = dxl <= (REAL)0 && dxr >= (REAL)0;
    int in_y = dyt <= (REAL)0 && dyb >= (REAL)0;
    if (in_x && in_y) return 1;
    REAL B2 = B + B;
    int have = 0;
    REAL qmin = 0;
    if (!in_x) {
        REAL ex = dxl > (REAL)0 ? dxl : dxr;
        REAL dys = -(B * ex) / C;
        dys = FMIN(FMAX(dys, dyt), dyb);
        REAL q = FMA(ex, FMA(B2, dys, A * ex), (C * dys) * dys);
        qmin = q; have = 1;
    }
    if (!in_y) {
        REAL ey = dyt > (REAL)0 ? dyt : dyb;
        REAL dxs = -(B * ey) / A;
        dxs = FMIN(FMAX(dxs, dxl), dxr);
        REAL q = FMA(dxs, FMA(B2, ey, A * dxs), (C * ey) * ey);
        if (!have || q < qmin) qmin = q;
    }
    return qmin <= Q;
}

/* Q of the Compact Box for opacity sigma; <= 0 means the Gaussian can never reach tau_alpha. */
static REAL FN(cb_threshold)(REAL sigma, const REAL *cfg)
{
    REAL ratio = sigma / CFG_AMIN(cfg);
    if (!(ratio > (REAL)1)) return (REAL)0;
    return CFG_CB_BETA(cfg) * ((REAL)2 * LOGC(ratio));
}

/*
 * Projection of one Gaussian (Sec. 3, Eqs. (2)-(3) and the text around them).
 * fp32 operation order (the contract the HIP path must reproduce bit for bit): every
 * expression below is evaluated exactly as written, left to right, with no fused ops.
 */
static void FN(project_one)(const REAL mu[3], const REAL s[3], const REAL q[4], REAL sigma, int deg,
                            const REAL *sh /* [(deg+1)^2][3] */, int width, int height,
                            const REAL *cam, const REAL *cfg, int tile, FN(proj) *o)
{
    const REAL *Rc = CAM_R(cam), *t0 = CAM_T(cam);
    const REAL fx = CAM_FX(cam), fy = CAM_FY(cam);
    memset(o, 0, sizeof(*o));

    /* viewing transformation W: camera-space mean */
    for (int i = 0; i < 3; i++)
        o->t[i] = Rc[3 * i + 0] * mu[0] + Rc[3 * i + 1] * mu[1] + Rc[3 * i + 2] * mu[2] + t0[i];
    if (!(o->t[2] > CFG_ZNEAR(cfg))) return;          /* behind / too close: culled        */

    /* Sigma_3D = R S S^T R^T  (Eq. (2)) */
    FN(quat_to_rot)(q, o->Rq);
    for (int i = 0; i < 3; i++)
        for (int j = 0; j < 3; j++) o->M[i][j] = o->Rq[i][j] * s[j];
    for (int i = 0; i < 3; i++)
        for (int j = 0; j < 3; j++)
            o->S3[i][j] = o->M[i][0] * o->M[j][0] + o->M[i][1] * o->M[j][1] + o->M[i][2] * o->M[j][2];

    /* J: Jacobian of the affine approximation of the projective map at t, with the usual
     * guard that the ratio t_x/t_z used INSIDE J is limited to a bit beyond the frustum.  */
    REAL tz = o->t[2];
    o->txz = o->t[0] / tz;
    o->tyz = o->t[1] / tz;
    o->cxz = o->txz; o->cyz = o->tyz; o->xin = 1; o->yin = 1;
    if (CFG_JCLAMP(cfg) > (REAL)0) {
        REAL limx = CFG_JCLAMP(cfg) * ((REAL)0.5 * (REAL)width / fx);
        REAL limy = CFG_JCLAMP(cfg) * ((REAL)0.5 * (REAL)height / fy);
        if (o->txz > limx) { o->cxz = limx; o->xin = 0; }
        if (o->txz < -limx) { o->cxz = -limx; o->xin = 0; }
        if (o->tyz > limy) { o->cyz = limy; o->yin = 0; }
        if (o->tyz < -limy) { o->cyz = -limy; o->yin = 0; }
    }
    REAL X = o->cxz * tz, Y = o->cyz * tz;
    REAL iz = (REAL)1 / tz;
    REAL iz2 = iz * iz;
    o->J00 = fx * iz;
    o->J02 = -(fx * X) * iz2;
    o->J11 = fy * iz;
    o->J12 = -(fy * Y) * iz2;

    /* Sigma' = J W Sigma_3D W^T J^T (Eq. (3)); marginalising along the viewing direction
     * keeps its upper-left 2x2 block, so only the first two rows of J are needed.          */
    for (int k = 0; k < 3; k++) {
        o->Tm[0][k] = o->J00 * Rc[0 + k] + o->J02 * Rc[6 + k];
        o->Tm[1][k] = o->J11 * Rc[3 + k] + o->J12 * Rc[6 + k];
    }
    REAL U[2][3];
    for (int i = 0; i < 2; i++)
        for (int k = 0; k < 3; k++)
            U[i][k] = o->Tm[i][0] * o->S3[0][k] + o->Tm[i][1] * o->S3[1][k] + o->Tm[i][2] * o->S3[2][k];
    REAL c00 = U[0][0] * o->Tm[0][0] + U[0][1] * o->Tm[0][1] + U[0][2] * o->Tm[0][2];
    REAL c01 = U[0][0] * o->Tm[1][0] + U[0][1] * o->Tm[1][1] + U[0][2] * o->Tm[1][2];
    REAL c11 = U[1][0] * o->Tm[1][0] + U[1][1] * o->Tm[1][1] + U[1][2] * o->Tm[1][2];
    o->a = c00 + CFG_LOWPASS(cfg);                   /* screen-space low-pass (dilation)  */
    o->b = c01;
    o->c = c11 + CFG_LOWPASS(cfg);
    o->det = o->a * o->c - o->b * o->b;
    if (!(o->det > (REAL)0)) return;
    REAL idet = (REAL)1 / o->det;
    o->conic[0] = o->c * idet;
    o->conic[1] = -o->b * idet;
    o->conic[2] = o->a * idet;

    o->mx = fx * o->txz + CAM_CX(cam);
    o->my = fy * o->tyz + CAM_CY(cam);
    int TX = (width + tile - 1) / tile, TY = (height + tile - 1) / tile;
    REAL inv_tile = (REAL)1 / (REAL)tile;            /* tile is a power of two: exact     */
    REAL hx, hy;                                     /* half-widths of the box around mu_2D */
    if (!CFG_CB(cfg)) {
        /* 3-sigma rule (Sec. 4.4): radius from the larger eigenvalue of Sigma_2D           */
        REAL mid = (REAL)0.5 * (o->a + o->c);
        REAL hd = (REAL)0.5 * (o->a - o->c);
        o->lam_max = mid + SQRT(hd * hd + o->b * o->b);
        o->radius = CEIL((REAL)3 * SQRT(o->lam_max));
        hx = hy = o->radius;
    } else {
        /* Compact Box: axis-aligned bounds of the ellipse q <= Q are sqrt(Q Sigma_xx), sqrt(Q Sigma_yy) */
        o->Q = FN(cb_threshold)(sigma, cfg);
        if (!(o->Q > (REAL)0)) return;
        hx = SQRT(o->Q * o->a);
        hy = SQRT(o->Q * o->c);
        o->radius = CEIL(hx > hy ? hx : hy);
    }
    if (!(hx < (REAL)1e6) || !(hy < (REAL)1e6) || !(FABS(o->mx) < (REAL)1e7) || !(FABS(o->my) < (REAL)1e7)) return;

    /* tiles met by the closed box [mu-h, mu+h]; tile (tx,ty) covers
     * [tile*tx, tile*tx+tile) x [tile*ty, ...)                                              */
    REAL fx0 = FLOOR((o->mx - hx) * inv_tile);
    REAL fy0 = FLOOR((o->my - hy) * inv_tile);
    REAL fx1 = FLOOR((o->mx + hx) * inv_tile) + (REAL)1;
    REAL fy1 = FLOOR((o->my + hy) * inv_tile) + (REAL)1;
    o->rect[0] = (int)FMIN(FMAX(fx0, (REAL)0), (REAL)TX);
    o->rect[1] = (int)FMIN(FMAX(fy0, (REAL)0), (REAL)TY);
    o->rect[2] = (int)FMIN(FMAX(fx1, (REAL)0), (REAL)TX);
    o->rect[3] = (int)FMIN(FMAX(fy1, (REAL)0), (REAL)TY);
    if ((o->rect[2] - o->rect[0]) * (o->rect[3] - o->rect[1]) <= 0) return;
    if (!CFG_CB(cfg)) {
        o->touched = (o->rect[2] - o->rect[0]) * (o->rect[3] - o->rect[1]);
    } else {
        /* within the box, only the tiles whose rectangle really meets the ellipse */
        o->touched = 0;
        for (int ty = o->rect[1]; ty < o->rect[3]; ty++)
            for (int tx = o->rect[0]; tx < o->rect[2]; tx++)
                o->touched += FN(cb_tile_hit)(o->mx, o->my, o->conic[0], o->conic[1], o->conic[2], o->Q, tx, ty, tile);
        if (o->touched == 0) return;
    }

    /* view-dependent colour: direction from the camera centre to the mean                  */
    REAL campos[3];
    for (int i = 0; i < 3; i++)
        campos[i] = -(Rc[0 + i] * t0[0] + Rc[3 + i] * t0[1] + Rc[6 + i] * t0[2]);
    for (int i = 0; i < 3; i++) o->dir[i] = mu[i] - campos[i];
    o->len = SQRT(o->dir[0] * o->dir[0] + o->dir[1] * o->dir[1] + o->dir[2] * o->dir[2]);
    for (int i = 0; i < 3; i++) o->d[i] = o->dir[i] / o->len;
    REAL Yb[16];
    FN(sh_basis)(o->d[0], o->d[1], o->d[2], Yb);
    int K = (deg + 1) * (deg + 1);
    for (int ch = 0; ch < 3; ch++) {
        REAL v = Yb[0] * sh[ch];
        for (int k = 1; k < K; k++) v = v + Yb[k] * sh[3 * k + ch];
        v = v + (REAL)0.5;
        o->clamped[ch] = v < (REAL)0;
        o->rgb[ch] = o->clamped[ch] ? (REAL)0 : v;
    }
    o->visible = 1;
}

/* Step a1: projection of all Gaussians.  Invisible ones get zeros everywhere. */
void FN(orc_preprocess)(int64_t n, int deg, const REAL *means, const REAL *scales, const REAL *quats,
                        const REAL *opac, const REAL *sh, int width, int height, const REAL *cam,
                        const REAL *cfg, int tile,
                        REAL *mean2d, REAL *depth, REAL *conic_opacity, REAL *rgb, int32_t *rect,
                        uint32_t *touched, uint8_t *clamped, int32_t *radius)
{
    int K = (deg + 1) * (deg + 1);
    for (int64_t i = 0; i < n; i++) {
        FN(proj) p;
        FN(project_one)(means + 3 * i, scales + 3 * i, quats + 4 * i, opac[i], deg, sh + 3 * K * i, width, height,
                        cam, cfg, tile, &p);
        if (!p.visible) {
            mean2d[2 * i] = mean2d[2 * i + 1] = 0; depth[i] = 0;
            for (int k = 0; k < 4; k++) { conic_opacity[4 * i + k] = 0; rect[4 * i + k] = 0; }
            for (int k = 0; k < 3; k++) { rgb[3 * i + k] = 0; clamped[3 * i + k] = 0; }
            touched[i] = 0; radius[i] = 0;
            continue;
        }
        mean2d[2 * i] = p.mx; mean2d[2 * i + 1] = p.my; depth[i] = p.t[2];
        conic_opacity[4 * i + 0] = p.conic[0]; conic_opacity[4 * i + 1] = p.conic[1];
        conic_opacity[4 * i + 2] = p.conic[2]; conic_opacity[4 * i + 3] = opac[i];
        for (int k = 0; k < 3; k++) { rgb[3 * i + k] = p.rgb[k]; clamped[3 * i + k] = (uint8_t)p.clamped[k]; }
        for (int k = 0; k < 4; k++) rect[4 * i + k] = p.rect[k];
        touched[i] = (uint32_t)p.touched;
        radius[i] = (int32_t)p.radius;
    }
}

/* Step a3 with the Compact Box: one (key, Gaussian) entry per tile of the Gaussian's box whose
 * rectangle meets its support ellipse, in Gaussian order, rows then columns (same key layout as the
 * 3-sigma emission).  depth_bits are the fp32 bit patterns of the depths. */
uint64_t FN(orc_emit_pairs_cb)(int64_t n, const int32_t *rect, const uint32_t *depth_bits, const REAL *mean2d,
                               const REAL *conic_opacity, const REAL *cfg, int TX, int tile,
                               uint64_t *keys, uint32_t *vals)
{
    uint64_t p = 0;
    for (int64_t i = 0; i < n; i++) {
        if (rect[4 * i + 2] <= rect[4 * i] || rect[4 * i + 3] <= rect[4 * i + 1]) continue;
        REAL Q = FN(cb_threshold)(conic_opacity[4 * i + 3], cfg);
        for (int ty = rect[4 * i + 1]; ty < rect[4 * i + 3]; ty++)
            for (int tx = rect[4 * i + 0]; tx < rect[4 * i + 2]; tx++) {
                if (!FN(cb_tile_hit)(mean2d[2 * i], mean2d[2 * i + 1], conic_opacity[4 * i], conic_opacity[4 * i + 1],
                                     conic_opacity[4 * i + 2], Q, tx, ty, tile))
                    continue;
                if (keys) {
                    keys[p] = ((uint64_t)(uint32_t)(ty * TX + tx) << 32) | depth_bits[i];
                    vals[p] = (uint32_t)i;
                }
                p++;
            }
    }
    return p;
}

/*
 * alpha_i(p) of Eq. (4)/(5) for one Gaussian at one pixel centre, with the blending
 * conventions: exponent must be <= 0, alpha is capped at alpha_max, and alphas below
 * alpha_min do not take part.  Returns 0 when the Gaussian does not take part.
 * fp32 order: dx = px - mx; dy = py - my; u = fma(2b, dy, a*dx); q = fma(dx, u, (c*dy)*dy);
 * power = -0.5*q; G = EXPNEG(power); alpha = min(alpha_max, sigma*G).
 */
static int FN(alpha_at)(REAL px, REAL py, REAL mx, REAL my, REAL ca, REAL cb, REAL cc, REAL sigma,
                        const REAL *cfg, REAL *alpha, REAL *dx_o, REAL *dy_o, REAL *G_o)
{
    REAL dx = px - mx, dy = py - my;
    REAL b2 = cb + cb;
    REAL u = FMA(b2, dy, ca * dx);
    REAL q = FMA(dx, u, (cc * dy) * dy);
    REAL power = (REAL)-0.5 * q;
    if (power > (REAL)0) return 0;
    REAL G = EXPNEG(power);
    REAL al = sigma * G;
    if (al > CFG_AMAX(cfg)) al = CFG_AMAX(cfg);
    if (al < CFG_AMIN(cfg)) return 0;
    *alpha = al; *dx_o = dx; *dy_o = dy; *G_o = G;
    return 1;
}

/*
 * Step a6: front-to-back alpha compositing of Eq. (4) for the pixels of the listed tiles.
 * A pixel stops consuming its list when the next transmittance T(1-alpha) would fall below
 * T_min (that Gaussian is NOT blended).  n_contrib = 1-based list position of the last
 * blended Gaussian (0 if none); final_T = T after it.  C += T*bg at the end.
 * fp32 order: w = alpha*T; C_ch = fma(rgb_ch, w, C_ch); T' = T*(1-alpha).
 */
void FN(orc_render_fwd)(const REAL *mean2d, const REAL *conic_opacity, const REAL *rgb,
                        const uint32_t *gauss_sorted, const uint32_t *ranges, int width, int height,
                        const REAL *cfg, int tile, const int32_t *tile_list, int n_tiles_listed,
                        REAL *image, REAL *final_T, uint32_t *n_contrib)
{
    int TX = (width + tile - 1) / tile, TY = (height + tile - 1) / tile;
    int ntl = tile_list ? n_tiles_listed : TX * TY;
    for (int it = 0; it < ntl; it++) {
        int tid = tile_list ? tile_list[it] : it;
        int tx = tid % TX, ty = tid / TX;
        uint32_t lo = ranges[2 * tid], hi = ranges[2 * tid + 1];
        for (int v = ty * tile; v < ty * tile + tile && v < height; v++)
            for (int u = tx * tile; u < tx * tile + tile && u < width; u++) {
                REAL px = (REAL)u + (REAL)0.5, py = (REAL)v + (REAL)0.5;
                REAL T = 1, C[3] = {0, 0, 0};
                uint32_t last = 0;
                for (uint32_t k = lo; k < hi; k++) {
                    uint32_t g = gauss_sorted[k];
                    REAL al, dx, dy, G;
                    if (!FN(alpha_at)(px, py, mean2d[2 * g], mean2d[2 * g + 1], conic_opacity[4 * g],
                                      conic_opacity[4 * g + 1], conic_opacity[4 * g + 2],
                                      conic_opacity[4 * g + 3], cfg, &al, &dx, &dy, &G))
                        continue;
                    REAL Tn = T * ((REAL)1 - al);
                    if (Tn < CFG_TMIN(cfg)) break;
                    REAL w = al * T;
                    for (int ch = 0; ch < 3; ch++) C[ch] = FMA(rgb[3 * g + ch], w, C[ch]);
                    T = Tn;
                    last = k - lo + 1;
                }
                size_t pix = (size_t)v * width + u;
                for (int ch = 0; ch < 3; ch++)
                    image[(size_t)ch * width * height + pix] = FMA(T, CFG_BG(cfg)[ch], C[ch]);
                final_T[pix] = T;
                n_contrib[pix] = last;
            }
    }
}

/*
 * Step a8: gradient of a scalar loss through Eq. (4), given dL/dC per pixel.
 * For the blended Gaussians 1..n of a pixel (front to back), with B_n = bg and
 * B_{i-1} = alpha_i c_i + (1 - alpha_i) B_i (the colour seen behind Gaussian i-1):
 *   dC/dc_i = alpha_i T_i ;  dC/dalpha_i = T_i (c_i - B_i).
 * alpha = min(alpha_max, sigma G): no gradient through the cap.  G = exp(-q/2),
 * q = a dx^2 + 2 b dx dy + c dy^2 with d = p - mu_2D.
 * Outputs (double accumulators): dL/dmu_2D [n,2], dL/dconic [n,3] (w.r.t. a, b, c as they
 * appear in q, b counted once with its factor 2), dL/dsigma [n], dL/drgb [n,3].
 */
void FN(orc_render_bwd)(const REAL *mean2d, const REAL *conic_opacity, const REAL *rgb,
                        const uint32_t *gauss_sorted, const uint32_t *ranges, int width, int height,
                        const REAL *cfg, int tile, const int32_t *tile_list, int n_tiles_listed,
                        const REAL *dL_dimage, double *d_mean2d, double *d_conic, double *d_opacity,
                        double *d_rgb, double *d_mean2d_abs /* may be NULL */)
{
    int TX = (width + tile - 1) / tile, TY = (height + tile - 1) / tile;
    int ntl = tile_list ? n_tiles_listed : TX * TY;
    size_t cap = 1024;
    struct contrib { uint32_t g; REAL al, T, dx, dy, G; } *list = malloc(cap * sizeof(*list));
    for (int it = 0; it < ntl; it++) {
        int tid = tile_list ? tile_list[it] : it;
        int tx = tid % TX, ty = tid / TX;
        uint32_t lo = ranges[2 * tid], hi = ranges[2 * tid + 1];
        if ((size_t)(hi - lo) > cap) { cap = hi - lo; list = realloc(list, cap * sizeof(*list)); }
        for (int v = ty * tile; v < ty * tile + tile && v < height; v++)
            for (int u = tx * tile; u < tx * tile + tile && u < width; u++) {
                REAL px = (REAL)u + (REAL)0.5, py = (REAL)v + (REAL)0.5;
                /* forward walk, remembering every blended Gaussian with its alpha and T */
                size_t m = 0;
                REAL T = 1;
                for (uint32_t k = lo; k < hi; k++) {
                    uint32_t g = gauss_sorted[k];
                    REAL al, dx, dy, G;
                    if (!FN(alpha_at)(px, py, mean2d[2 * g], mean2d[2 * g + 1], conic_opacity[4 * g],
                                      conic_opacity[4 * g + 1], conic_opacity[4 * g + 2],
                                      conic_opacity[4 * g + 3], cfg, &al, &dx, &dy, &G))
                        continue;
                    REAL Tn = T * ((REAL)1 - al);
                    if (Tn < CFG_TMIN(cfg)) break;
                    list[m].g = g; list[m].al = al; list[m].T = T; list[m].dx = dx; list[m].dy = dy;
                    list[m].G = G; m++;
                    T = Tn;
                }
                size_t pix = (size_t)v * width + u;
                REAL dC[3];
                for (int ch = 0; ch < 3; ch++) dC[ch] = dL_dimage[(size_t)ch * width * height + pix];
                REAL B[3] = {CFG_BG(cfg)[0], CFG_BG(cfg)[1], CFG_BG(cfg)[2]};
                for (size_t r = m; r-- > 0;) {
                    uint32_t g = list[r].g;
                    REAL al = list[r].al, Ti = list[r].T, dx = list[r].dx, dy = list[r].dy, G = list[r].G;
                    REAL dL_dal = 0;
                    for (int ch = 0; ch < 3; ch++) {
                        d_rgb[3 * g + ch] += (double)(al * Ti * dC[ch]);
                        dL_dal += Ti * (rgb[3 * g + ch] - B[ch]) * dC[ch];
                        B[ch] = al * rgb[3 * g + ch] + ((REAL)1 - al) * B[ch];
                    }
                    REAL sigma = conic_opacity[4 * g + 3];
                    if (sigma * G > CFG_AMAX(cfg)) continue;      /* capped: alpha is constant */
                    d_opacity[g] += (double)(G * dL_dal);
                    REAL dL_dG = sigma * dL_dal;
                    REAL dL_dq = (REAL)-0.5 * G * dL_dG;          /* G = exp(-q/2)             */
                    REAL ca = conic_opacity[4 * g], cb = conic_opacity[4 * g + 1], cc = conic_opacity[4 * g + 2];
                    d_conic[3 * g + 0] += (double)(dL_dq * dx * dx);
                    d_conic[3 * g + 1] += (double)(dL_dq * (REAL)2 * dx * dy);
                    d_conic[3 * g + 2] += (double)(dL_dq * dy * dy);
                    /* d = p - mu  =>  dq/dmu = -(2 a dx + 2 b dy, 2 b dx + 2 c dy) */
                    REAL gmx = -dL_dq * ((REAL)2 * ca * dx + (REAL)2 * cb * dy);
                    REAL gmy = -dL_dq * ((REAL)2 * cb * dx + (REAL)2 * cc * dy);
                    d_mean2d[2 * g + 0] += (double)gmx;
                    d_mean2d[2 * g + 1] += (double)gmy;
                    /* absolute positional gradient (the supplement's implementation details adopt it for
                     * splitting): every pixel's contribution enters with its magnitude, component-wise,
                     * so that contributions of opposite sign do not cancel */
                    if (d_mean2d_abs) {
                        d_mean2d_abs[2 * g + 0] += (double)FABS(gmx);
                        d_mean2d_abs[2 * g + 1] += (double)FABS(gmy);
                    }
                }
            }
    }
    free(list);
}

/*
 * Step a9: chain the screen-space gradients of one view back to the Gaussian parameters
 * through the projection (reverse of project_one, same intermediate names).
 * d_conic is w.r.t. (conic0, conic1, conic2) as used in q (conic1 multiplied by 2 there).
 * Outputs are OVERWRITTEN.  Invisible Gaussians get zero gradients.
 */
void FN(orc_preprocess_bwd)(int64_t n, int deg, const REAL *means, const REAL *scales, const REAL *quats,
                            const REAL *opac, const REAL *sh, int width, int height, const REAL *cam, const REAL *cfg,
                            int tile, const double *d_mean2d, const double *d_conic,
                            const double *d_opacity_in, const double *d_rgb,
                            double *d_means, double *d_scales, double *d_quats, double *d_opac,
                            double *d_sh)
{
    int K = (deg + 1) * (deg + 1);
    const REAL *Rc = CAM_R(cam);
    const REAL fx = CAM_FX(cam), fy = CAM_FY(cam);
    for (int64_t i = 0; i < n; i++) {
        double *gm = d_means + 3 * i, *gs = d_scales + 3 * i, *gq = d_quats + 4 * i, *gsh = d_sh + 3 * K * i;
        for (int k = 0; k < 3; k++) gm[k] = gs[k] = 0;
        for (int k = 0; k < 4; k++) gq[k] = 0;
        for (int k = 0; k < 3 * K; k++) gsh[k] = 0;
        d_opac[i] = 0;
        FN(proj) p;
        FN(project_one)(means + 3 * i, scales + 3 * i, quats + 4 * i, opac[i], deg, sh + 3 * K * i, width, height,
                        cam, cfg, tile, &p);
        if (!p.visible) continue;
        d_opac[i] = d_opacity_in[i];

        /* ---- colour: rgb = max(0, 0.5 + sum_k Y_k(d) c_k) ---- */
        double Yb[16]; REAL Ybr[16], dYr[16][3];
        FN(sh_basis)(p.d[0], p.d[1], p.d[2], Ybr);
        FN(sh_basis_grad)(p.d[0], p.d[1], p.d[2], dYr);
        for (int k = 0; k < 16; k++) Yb[k] = Ybr[k];
        double g_d[3] = {0, 0, 0};
        for (int ch = 0; ch < 3; ch++) {
            if (p.clamped[ch]) continue;
            double g = d_rgb[3 * i + ch];
            for (int k = 0; k < K; k++) {
                gsh[3 * k + ch] = g * Yb[k];
                for (int ax = 0; ax < 3; ax++) g_d[ax] += g * (double)sh[3 * K * i + 3 * k + ch] * (double)dYr[k][ax];
            }
        }
        /* d = dir/|dir|  =>  g_dir = (g_d - d (d . g_d)) / |dir| */
        double dot = g_d[0] * p.d[0] + g_d[1] * p.d[1] + g_d[2] * p.d[2];
        for (int ax = 0; ax < 3; ax++) gm[ax] += (g_d[ax] - (double)p.d[ax] * dot) / (double)p.len;

        /* ---- conic = Sigma_2D^-1 -> (a, b, c) ---- */
        double a = p.a, b = p.b, c = p.c, det = p.det;
        double g0 = d_conic[3 * i], g1 = d_conic[3 * i + 1], g2 = d_conic[3 * i + 2];
        /* conic0 = c/det, conic1 = -b/det, conic2 = a/det, det = a c - b^2 */
        double g_det = -(g0 * c - g1 * b + g2 * a) / (det * det);
        double g_a = g2 / det + g_det * c;
        double g_b = -g1 / det + g_det * (-2 * b);
        double g_c = g0 / det + g_det * a;
        /* Sigma_2D (without low-pass) = Tm S3 Tm^T; a=cov00, b=cov01=cov10, c=cov11 */
        double Gc[2][2] = {{g_a, 0.5 * g_b}, {0.5 * g_b, g_c}};
        double g_S3[3][3], g_Tm[2][3];
        for (int r = 0; r < 3; r++)
            for (int s = 0; s < 3; s++) {
                double v = 0;
                for (int x = 0; x < 2; x++)
                    for (int y = 0; y < 2; y++) v += (double)p.Tm[x][r] * Gc[x][y] * (double)p.Tm[y][s];
                g_S3[r][s] = v;
            }
        for (int x = 0; x < 2; x++)
            for (int r = 0; r < 3; r++) {
                double v = 0;
                for (int y = 0; y < 2; y++)
                    for (int s = 0; s < 3; s++) v += 2 * Gc[x][y] * (double)p.Tm[y][s] * (double)p.S3[s][r];
                g_Tm[x][r] = v;
            }
        /* Tm = J Rc, J = [[J00,0,J02],[0,J11,J12]] */
        double g_J00 = 0, g_J02 = 0, g_J11 = 0, g_J12 = 0;
        for (int k = 0; k < 3; k++) {
            g_J00 += g_Tm[0][k] * Rc[0 + k];
            g_J02 += g_Tm[0][k] * Rc[6 + k];
            g_J11 += g_Tm[1][k] * Rc[3 + k];
            g_J12 += g_Tm[1][k] * Rc[6 + k];
        }
        /* J00 = fx iz, J02 = -fx X iz^2, J11 = fy iz, J12 = -fy Y iz^2; X = cxz tz, Y = cyz tz; iz = 1/tz */
        double tz = p.t[2], iz = 1.0 / tz, iz2 = iz * iz;
        double X = (double)p.cxz * tz, Yv = (double)p.cyz * tz;
        double g_iz = fx * g_J00 + fy * g_J11 - 2 * fx * X * iz * g_J02 - 2 * fy * Yv * iz * g_J12;
        double g_X = -fx * iz2 * g_J02, g_Y = -fy * iz2 * g_J12;
        double g_t[3] = {0, 0, 0};
        double g_txz = 0, g_tyz = 0;
        g_t[2] += g_X * p.cxz + g_Y * p.cyz - g_iz * iz2;
        if (p.xin) g_txz += g_X * tz;
        if (p.yin) g_tyz += g_Y * tz;
        /* mu_2D = (fx txz + cx, fy tyz + cy) */
        g_txz += fx * d_mean2d[2 * i];
        g_tyz += fy * d_mean2d[2 * i + 1];
        /* txz = tx/tz, tyz = ty/tz */
        g_t[0] += g_txz * iz;
        g_t[1] += g_tyz * iz;
        g_t[2] += -(g_txz * p.t[0] + g_tyz * p.t[1]) * iz2;
        /* t = Rc mu + t0 */
        for (int ax = 0; ax < 3; ax++)
            gm[ax] += Rc[0 + ax] * g_t[0] + Rc[3 + ax] * g_t[1] + Rc[6 + ax] * g_t[2];

        /* ---- Sigma_3D = M M^T, M = Rq diag(s) ---- */
        double g_M[3][3];
        for (int r = 0; r < 3; r++)
            for (int s = 0; s < 3; s++) {
                double v = 0;
                for (int k = 0; k < 3; k++) v += (g_S3[r][k] + g_S3[k][r]) * (double)p.M[k][s];
                g_M[r][s] = v;
            }
        double g_R[3][3];
        for (int r = 0; r < 3; r++)
            for (int s = 0; s < 3; s++) {
                gs[s] += g_M[r][s] * (double)p.Rq[r][s];
                g_R[r][s] = g_M[r][s] * (double)scales[3 * i + s];
            }
        /* Rq(w,x,y,z): differentiate each entry of quat_to_rot */
        double w = quats[4 * i], x = quats[4 * i + 1], y = quats[4 * i + 2], z = quats[4 * i + 3];
        gq[0] = 2 * (-z * g_R[0][1] + y * g_R[0][2] + z * g_R[1][0] - x * g_R[1][2] - y * g_R[2][0] + x * g_R[2][1]);
        gq[1] = 2 * (y * g_R[0][1] + z * g_R[0][2] + y * g_R[1][0] - 2 * x * g_R[1][1] - w * g_R[1][2]
                     + z * g_R[2][0] + w * g_R[2][1] - 2 * x * g_R[2][2]);
        gq[2] = 2 * (-2 * y * g_R[0][0] + x * g_R[0][1] + w * g_R[0][2] + x * g_R[1][0] + z * g_R[1][2]
                     - w * g_R[2][0] + z * g_R[2][1] - 2 * y * g_R[2][2]);
        gq[3] = 2 * (-2 * z * g_R[0][0] - w * g_R[0][1] + x * g_R[0][2] + w * g_R[1][0] - 2 * z * g_R[1][1]
                     + y * g_R[1][2] + x * g_R[2][0] + y * g_R[2][1]);
    }
}

/* Step a7: L = mean over 3*H*W of |C - G| (the L1 term of Sec. 4.5); dL/dC = sign(C-G)/(3HW). */
double FN(orc_l1)(const REAL *image, const REAL *target, int width, int height, REAL *dL_dimage)
{
    size_t m = (size_t)3 * width * height;
    REAL scale = (REAL)1 / (REAL)m;
    double loss = 0;
    for (size_t k = 0; k < m; k++) {
        REAL d = image[k] - target[k];
        loss += (double)FABS(d);
        if (dL_dimage) dL_dimage[k] = d > 0 ? scale : (d < 0 ? -scale : (REAL)0);
    }
    return loss / (double)m;
}

/*
 * Step a10: per-pixel error e = mean over channels of |r - g| (Sec. 4.2, first equation),
 * then a scalar threshold t and the mask e > t (third equation).
 *   rule 0: t = mean(e) + k * std(e), population std, two-pass, double accumulators,
 *           rounded once to REAL (the benchmark's rule);
 *   rule 1: t = min(e) + k * (max(e) - min(e)), i.e. min-max normalised e > k (the paper's
 *           second and third equations), in REAL.
 * fp32 order: e = ((|d0| + |d1|) + |d2|) / 3.
 */
REAL FN(orc_error_mask)(const REAL *image, const REAL *target, int width, int height, int rule, REAL k,
                        uint8_t *mask, REAL *err_out)
{
    size_t m = (size_t)width * height;
    REAL *e = err_out ? err_out : malloc(m * sizeof(REAL));
    for (size_t p = 0; p < m; p++) {
        REAL d0 = FABS(image[p] - target[p]);
        REAL d1 = FABS(image[m + p] - target[m + p]);
        REAL d2 = FABS(image[2 * m + p] - target[2 * m + p]);
        e[p] = ((d0 + d1) + d2) / (REAL)3;
    }
    REAL thr;
    if (rule == 0) {
        double s = 0, s2 = 0;
        for (size_t p = 0; p < m; p++) s += (double)e[p];
        double mean = s / (double)m;
        for (size_t p = 0; p < m; p++) { double d = (double)e[p] - mean; s2 += d * d; }
        thr = (REAL)(mean + (double)k * sqrt(s2 / (double)m));
    } else {
        REAL lo = e[0], hi = e[0];
        for (size_t p = 1; p < m; p++) { if (e[p] < lo) lo = e[p]; if (e[p] > hi) hi = e[p]; }
        thr = lo + k * (hi - lo);
    }
    for (size_t p = 0; p < m; p++) mask[p] = e[p] > thr;
    if (!err_out) free(e);
    return thr;
}

/*
 * Step a11: the inner double sum of the densification score (Sec. 4.2, Eq. for s_d) for ONE
 * view: for every Gaussian, the number of mask pixels it contributes to.  The footprint
 * Omega_i is read as "pixels where the Gaussian is blended by the forward pass":
 *   score_mode 0 (WEIGHT): blended and blending weight alpha_i T_i > alpha_min;
 *   score_mode 1 (ALPHA):  blended (alpha_i >= alpha_min before the pixel terminated).
 * counts are ACCUMULATED (sum over views is the caller's loop; s_d = counts / K).
 */
void FN(orc_score)(const REAL *mean2d, const REAL *conic_opacity, const uint32_t *gauss_sorted,
                   const uint32_t *ranges, int width, int height, const REAL *cfg, int tile,
                   int score_mode, const uint8_t *mask, const int32_t *tile_list, int n_tiles_listed,
                   int32_t *counts)
{
    int TX = (width + tile - 1) / tile, TY = (height + tile - 1) / tile;
    int ntl = tile_list ? n_tiles_listed : TX * TY;
    for (int it = 0; it < ntl; it++) {
        int tid = tile_list ? tile_list[it] : it;
        int tx = tid % TX, ty = tid / TX;
        uint32_t lo = ranges[2 * tid], hi = ranges[2 * tid + 1];
        for (int v = ty * tile; v < ty * tile + tile && v < height; v++)
            for (int u = tx * tile; u < tx * tile + tile && u < width; u++) {
                if (!mask[(size_t)v * width + u]) continue;
                REAL px = (REAL)u + (REAL)0.5, py = (REAL)v + (REAL)0.5;
                REAL T = 1;
                for (uint32_t k = lo; k < hi; k++) {
                    uint32_t g = gauss_sorted[k];
                    REAL al, dx, dy, G;
                    if (!FN(alpha_at)(px, py, mean2d[2 * g], mean2d[2 * g + 1], conic_opacity[4 * g],
                                      conic_opacity[4 * g + 1], conic_opacity[4 * g + 2],
                                      conic_opacity[4 * g + 3], cfg, &al, &dx, &dy, &G))
                        continue;
                    REAL Tn = T * ((REAL)1 - al);
                    if (Tn < CFG_TMIN(cfg)) break;
                    REAL w = al * T;
                    if (score_mode == 1 || w > CFG_AMIN(cfg)) counts[g] += 1;
                    T = Tn;
                }
            }
    }
}

/* Number of (Gaussian, pixel) alpha evaluations the forward pass of the listed tiles makes
 * (list entries examined, including skipped ones and the one that terminates a pixel).     */
int64_t FN(orc_count_evals)(const REAL *mean2d, const REAL *conic_opacity, const uint32_t *gauss_sorted,
                            const uint32_t *ranges, int width, int height, const REAL *cfg, int tile,
                            const int32_t *tile_list, int n_tiles_listed)
{
    int TX = (width + tile - 1) / tile, TY = (height + tile - 1) / tile;
    int ntl = tile_list ? n_tiles_listed : TX * TY;
    int64_t total = 0;
    for (int it = 0; it < ntl; it++) {
        int tid = tile_list ? tile_list[it] : it;
        int tx = tid % TX, ty = tid / TX;
        uint32_t lo = ranges[2 * tid], hi = ranges[2 * tid + 1];
        for (int v = ty * tile; v < ty * tile + tile && v < height; v++)
            for (int u = tx * tile; u < tx * tile + tile && u < width; u++) {
                REAL px = (REAL)u + (REAL)0.5, py = (REAL)v + (REAL)0.5;
                REAL T = 1;
                for (uint32_t k = lo; k < hi; k++) {
                    uint32_t g = gauss_sorted[k];
                    REAL al, dx, dy, G;
                    total++;
                    if (!FN(alpha_at)(px, py, mean2d[2 * g], mean2d[2 * g + 1], conic_opacity[4 * g],
                                      conic_opacity[4 * g + 1], conic_opacity[4 * g + 2],
                                      conic_opacity[4 * g + 3], cfg, &al, &dx, &dy, &G))
                        continue;
                    REAL Tn = T * ((REAL)1 - al);
                    if (Tn < CFG_TMIN(cfg)) break;
                    T = Tn;
                }
            }
    }
    return total;
}
