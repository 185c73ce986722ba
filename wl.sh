#!/bin/bash
cd $GRAFT_REPO_ROOT/_work/gb2
for rep in 1 2; do
for v in w_nn192_42 w_nn192_24 w_nn256_24; do
  NCOPY=3 timeout -k 5 60 ./$v 2048 12288 7022 1 0 200 || exit 1
  NCOPY=3 timeout -k 5 60 ./$v 2048 12288 5376 1 0 200 || exit 1
done
done
